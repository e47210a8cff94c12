/* scars.h -- C ABI of the MI355X (gfx950) skew-aware cached embedding-bag library.
 *
 * The library implements, for ONE GPU's share of a recommendation-model batch, the embedding step
 * of the communication-avoiding scheme of "Stochastic Communication Avoidance for Recommendation
 * Systems" (arxiv 2411.01611): embedding tables live in (pinned) host memory (Section II, Fig. 1);
 * a skew table over all embeddings is built and its top entries are kept on the device under a
 * byte budget (Section III, Section IV); lookups that fall in that cached set C cost no transfer
 * (Section II-B, eq. (6)), the rest are fetched over the host link; the backward pass aggregates
 * the gradient per embedding and applies one optimizer step, hot rows on the device and cold rows
 * in host memory (Section IV, discussion of Tables 1-4).
 *
 * Conventions
 *  - T tables, rows[t] rows each, N = sum rows < 2^31.  Global row id  gid = row_base[t] + idx,
 *    row_base = exclusive prefix sum of rows.  D = dim (same for all tables), row bytes
 *    R = D * (4 for fp32 | 2 for bf16); R % 16 == 0 and R <= 1024.
 *  - A batch is "jagged, table-major": offsets has T*B+1 int32 entries, offsets[0] = 0,
 *    offsets[T*B] = L; bag g = t*B + b owns lookups [offsets[g], offsets[g+1]); indices[L] are
 *    table-local int32 row ids.  One lookup per (sample, table) is the case offsets[g] = g.
 *  - "DEVICE" pointers are HIP device memory, "HOST" pointers ordinary host memory, "PINNED" host
 *    memory allocated with hipHostMalloc (device-mapped).  The caller owns every buffer; the
 *    library allocates no device memory and frees nothing it is given.  Buffers must stay alive
 *    until the stream work that uses them has finished.
 *  - Every call returns SCARS_OK (0) or a negative error code and never throws.  Work is enqueued
 *    on the caller's stream (a hipStream_t passed as void*; NULL = the default stream) and the
 *    call returns without waiting unless stated.  Calls on one handle must be issued in stream
 *    order; two calls on one handle must not run concurrently.
 *  - Some options (SCARS_TUNE_PRESORT, SCARS_TUNE_LOOKAHEAD) run part of a call on up to two streams the library
 *    owns (default priority, non-blocking, created by the first scars_bind_buffers on a handle, always joined back
 *    into the caller's stream before the results are needed).  They only overlap with the caller's stream if they sit
 *    on other hardware queues: a process has few (4 by default), handed out as streams are created, so bind a
 *    handle's buffers before creating many streams of your own.  SCARS_COUNTER_AHEAD_NOT_OVERLAPPED tells, in profile
 *    mode, when such an overlap did not happen.
 *  - Two errors are detected on the device and latched in the handle's status word, to be read by
 *    scars_sync_status: SCARS_ERR_INDEX_RANGE (an index < 0 or >= rows[t]: that lookup is treated
 *    as absent everywhere -- not counted, neither hit nor miss, adds nothing, updates nothing) and
 *    SCARS_ERR_OFFSETS (offsets not starting at 0, not ending at L, or decreasing: outputs of that
 *    call are unspecified, but every memory access stays inside the bound buffers).
 */
#ifndef SCARS_H
#define SCARS_H
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SCARS_OK 0
#define SCARS_ERR_INVALID_ARG (-1)
#define SCARS_ERR_NOT_BUILT (-2)   /* remap / fwd / bwd / flush before a build_cache that selected a hot set */
#define SCARS_ERR_WORKSPACE (-3)   /* bound buffers too small for the request, or nothing bound */
#define SCARS_ERR_HIP (-4)         /* a HIP runtime call failed; text in scars_last_error */
#define SCARS_ERR_INDEX_RANGE (-5) /* device-detected, latched */
#define SCARS_ERR_OFFSETS (-6)     /* device-detected, latched */

#define SCARS_DTYPE_F32 0
#define SCARS_DTYPE_BF16 1
#define SCARS_OPT_SGD 0
#define SCARS_OPT_ADAGRAD 1

#define SCARS_MAX_TABLES 1024
#define SCARS_MAX_ROW_BYTES 1024

typedef struct scars_handle scars_handle;

/* Problem statement (Section II: tables in main memory; Section IV: optimizer stage). */
typedef struct {
    int32_t num_tables;        /* T, 1..SCARS_MAX_TABLES */
    const int64_t* rows;       /* HOST [T], each >= 1, sum < 2^31 */
    int32_t dim;               /* D */
    int32_t dtype;             /* SCARS_DTYPE_*: storage type of rows; sums are always fp32 */
    void* const* host_tables;  /* HOST [T] of PINNED pointers, table t row-major [rows[t]][D] */
    int32_t optimizer;         /* SCARS_OPT_* */
    float* const* host_state;  /* HOST [T] of PINNED fp32 [rows[t]][D] Adagrad accumulators; NULL for SGD */
} scars_config;

/* Launch tuning; results never depend on it (integer outputs bit for bit; floating-point ones too, except where a
 * tuning's comment says that the order of an fp64 sum changes).  The ordered compactions (hit/miss lists, run starts, sample lists)
 * count per tile of 2048 items, then need each tile's start: with few tiles the writing kernel adds up the counts
 * of the tiles before its own, beyond the limit a separate scan kernel runs first.  A limit of 0 always scans. */
#define SCARS_TUNE_FUSED_SCAN_MAX_TILES 1       /* default 4096, which is also the most */
/* Value n > 0: for batches of at least n lookups, when the cache is smaller than the tables, scars_remap also starts
 * the integer half of the backward pass of the same batch (pairs, sort, run starts; it needs the remap outputs only)
 * on a stream the library owns (default priority, created by scars_bind_buffers), so that it runs while
 * scars_embedding_bag_fwd waits on the host link for the missed rows.  scars_embedding_bag_bwd_update makes the
 * caller's stream wait for it and uses it when it is called for that batch (same remap_out arrays, offsets, L and
 * B), after that batch's forward pass, and without a scars_bwd_out; otherwise it sorts again itself.  The next call
 * of remap, build_cache, sync_status or bwd_update waits for outstanding side-stream work first.  For the same
 * batches bwd_update also runs its long-run kernels (HBM-bound) on that stream beside the per-row kernel (bound by
 * the host link while it writes cold rows) and joins them before it returns; and scars_embedding_bag_fwd, when bags
 * hold one lookup on average, pools the bags that need no fetched row on a further stream beside the fetch of the
 * missed rows, joined before it returns.  The two
 * cross-stream waits cost some 10-20 us per step: not worth it for small batches.  Under HIP graph capture the side
 * stream joins the capture: end the capture after the bwd_update (or sync_status) that joins it back.  Default 0. */
#define SCARS_TUNE_PRESORT 2
/* Batches of at most this many lookups sum the long runs (more than 64 lookups of one row) and update the other rows
 * in one launch of the backward pass instead of two: the two jobs touch disjoint rows, and sharing a launch hides the
 * shorter one's chain of dependent memory round trips.  Not used while SCARS_TUNE_PRESORT runs the long runs on the
 * side stream.  0 = never (two launches). */
#define SCARS_TUNE_FUSED_LONG_MAX_L 3           /* default 2^31 - 1: every batch */
/* Non-zero: scars_remap also writes the (row, bag) pairs that the backward pass of the same batch sorts, in the
 * launch that lists hits and misses (8 more bytes written per lookup; a backward pass called with the same remap
 * outputs, offsets, L and B then starts at its sort).  0: the backward pass builds them itself, as it does anyway
 * when unique_miss_gid is set or another batch was remapped in between. */
#define SCARS_TUNE_PAIRS_IN_REMAP 4             /* default 1 */
/* Most workgroups the per-row update kernel of the backward pass is launched with (it strides over the rows, so any
 * value gives the same results).  While it writes cold rows it holds its compute units' memory queues full of host
 * requests, and kernels of other streams that share those units crawl; a few hundred workgroups still saturate the
 * host link and leave room for them. */
/* At most 65536; default 0: 8192 with every row cached, else 1024 (768 for rows of 512 bytes or more; while rows are
 * fetched ahead 4096 for rows of 128 bytes or less). */
#define SCARS_TUNE_UPDATE_MAX_BLOCKS 5
/* Non-zero: scars_remap may be called for the next batch before scars_embedding_bag_bwd_update of the current one (it
 * then leaves alone everything that update uses: it writes no pairs and starts no preparation), and
 * scars_embedding_bag_bwd_update_ahead is allowed:
 * with SCARS_TUNE_PRESORT set, that call prepares the next batch's sorted segments on the library's side stream while
 * its own update runs (also when every row is cached and there is nothing to fetch).  The two batches need remap
 * outputs of their own. */
#define SCARS_TUNE_LOOKAHEAD 6                  /* default 0 */
/* Non-zero: scars_embedding_bag_bwd_update_ahead carries the fetch of the next batch's rows in the first workgroups
 * of its own update launch, on the caller's stream, whenever the update is one launch (see
 * SCARS_TUNE_FUSED_LONG_MAX_L); the two directions of the host link then overlap without a second hardware queue.
 * 0: the fetch is a launch of its own on the library's second stream. */
#define SCARS_TUNE_FUSED_FETCH 7                /* default 1 */
/* Value n > 0: the caller states that in every batch each table gets at most n lookups (offsets[(t+1)*B] -
 * offsets[t*B] <= n; one index per sample and table with B <= n is the usual case).  For n <= 4096 (and up to 256
 * tables) the backward pass then sorts each table's (row, bag) pairs by itself, one workgroup per table in LDS, and
 * lists the run starts in a second launch: two launches instead of three per radix pass and two more; the results
 * are the same.  A scars_embedding_bag_bwd_update that is not asked for its sorted segments (no scars_bwd_out), outside
 * the look-ahead order, needs no list of runs at all: the sorting workgroup leaves each run's length and row at the
 * run's first position and the update goes by position, in one launch; runs of more than 64 lookups are then summed
 * whole by one workgroup each (they cannot be longer than n), in fp64 as always but in another order than the general
 * path's, so the updated rows of the two can differ in the last bit of a rounding.  When scars_remap has left the batch's pairs for the backward pass (SCARS_TUNE_PAIRS_IN_REMAP) and
 * rows can be cold, scars_embedding_bag_fwd of the same batch carries the sort in the first workgroups of the launch
 * that fetches the missed rows, and scars_embedding_bag_bwd_update finds it done if it is the next call that sorts.
 * A batch that breaks the statement latches SCARS_ERR_OFFSETS (reported by scars_sync_status) and its backward
 * results are unspecified (all accesses stay in bounds).
 * 0 (default): nothing is assumed. */
#define SCARS_TUNE_MAX_TABLE_LOOKUPS 8

/* Host-side counters (never reset); -1 for an unknown counter. */
#define SCARS_COUNTER_PREPARED_USED 1  /* bwd_update calls that used the segments prepared under SCARS_TUNE_PRESORT */
#define SCARS_COUNTER_AHEAD_USED 2     /* forward passes that found their missed rows fetched ahead */
/* Self-check of the overlap the library's own streams are for (only counted while scars_profile_enable is on, at
 * scars_profile_read): updates that had the next batch's fetch enqueued beside them on the library's second stream,
 * and how many of those fetches did NOT run at the same time as the update (less than a quarter of the shorter one
 * overlapped): a sign that the library's stream shares a hardware queue with the caller's. */
#define SCARS_COUNTER_AHEAD_TIMED 3
#define SCARS_COUNTER_AHEAD_NOT_OVERLAPPED 4
#define SCARS_COUNTER_SORTED_IN_FWD_USED 5 /* bwd_update calls whose per-table sort (SCARS_TUNE_MAX_TABLE_LOOKUPS) the forward pass had done */
int64_t scars_get_counter(const scars_handle* h, int32_t which);
int32_t scars_set_tuning(scars_handle* h, int32_t which, int64_t value);

/* Sizes, in bytes, of the DEVICE buffers the caller must allocate (all 256-byte aligned). */
typedef struct {
    int64_t k;                  /* rows the budget buys: min(N, floor(budget_bytes / R)) */
    int64_t counts_bytes;       /* uint32 [N]  skew table */
    int64_t slot_of_bytes;      /* int32  [N]  gid -> cache slot or -1 */
    int64_t hot_gid_bytes;      /* int32  [k]  slot -> gid, hottest first */
    int64_t cache_bytes;        /* [k][D] rows in the tables' dtype */
    int64_t state_cache_bytes;  /* fp32 [k][D] Adagrad accumulators of cached rows; 0 for SGD */
    int64_t workspace_bytes;    /* scratch: descriptors, status word, selection and sort buffers,
                                   staging area for rows fetched over the host link (max_L rows) */
    /* per-batch outputs at max_L lookups / max_G bags */
    int64_t per_lookup_bytes;   /* int32 [max_L]: slot, gid, loc, hit_pos, miss_pos, miss_gid, sorted_gid, sorted_bag, unique_gid */
    int64_t seg_start_bytes;    /* int32 [max_L + 1] */
    int64_t out_bytes;          /* fp32 [max_G][D] */
} scars_sizes;

typedef struct {
    uint32_t* counts;     /* DEVICE */
    int32_t* slot_of;     /* DEVICE */
    int32_t* hot_gid;     /* DEVICE */
    void* cache;          /* DEVICE */
    float* state_cache;   /* DEVICE, NULL for SGD */
    void* workspace;      /* DEVICE */
    int64_t budget_bytes; /* the three arguments scars_query_sizes was called with */
    int64_t max_L;
    int64_t max_G;
    /* how many bytes each buffer above really has; scars_bind_buffers returns SCARS_ERR_WORKSPACE when one is
     * smaller than scars_query_sizes asks for with these three arguments (a buffer that may be NULL may say 0) */
    int64_t counts_bytes, slot_of_bytes, hot_gid_bytes, cache_bytes, state_cache_bytes, workspace_bytes;
} scars_buffers;

/* Outputs of scars_remap, all DEVICE, each int32 [L] unless noted. */
typedef struct {
    int32_t* slot;        /* slot_of[gid_i], -1 for a miss or an invalid lookup */
    int32_t* gid;         /* global row id, -1 for an invalid lookup */
    int32_t* loc;         /* where forward reads the row: slot for a hit, k + (rank in the miss list) for a miss, -1 invalid */
    int32_t* hit_pos;     /* positions i with slot >= 0, ascending; first n_hit entries valid */
    int32_t* miss_pos;    /* positions of misses, ascending; first n_miss entries valid */
    int32_t* miss_gid;    /* gid of each miss, same order as miss_pos */
    int32_t* n_hit_miss;  /* int32 [2] = {n_hit, n_miss} */
    /* Optional coalescing (Section II-A: send each distinct embedding of the batch once, plus per-lookup indices).
     * Both NULL: one staged row per missed lookup, loc as above.  Both set: unique_miss_gid [L] receives the
     * distinct missed gids in ascending order (first n_unique_miss[0] entries), n_unique_miss int32 [2] =
     * {U_miss, n_miss}, and loc of a miss = k + (index of its gid in unique_miss_gid): forward then fetches each
     * distinct cold row once over the host link. */
    int32_t* unique_miss_gid;
    int32_t* n_unique_miss;
} scars_remap_out;

/* Optional outputs of scars_embedding_bag_bwd_update, all DEVICE. */
typedef struct {
    int32_t* sorted_gid;  /* [L] gids of valid lookups ordered by (gid, position); first n_valid entries */
    int32_t* sorted_bag;  /* [L] bag of each sorted lookup */
    int32_t* seg_start;   /* [L+1] first sorted position of each distinct gid; seg_start[U] = n_valid */
    int32_t* unique_gid;  /* [L] distinct gids ascending; first U entries */
    int32_t* n_unique;    /* int32 [2] = {U, n_valid} */
} scars_bwd_out;

/* Outputs of scars_classify_samples, all DEVICE int32. */
typedef struct {
    int32_t* is_hot;        /* [B] 1 if every lookup of the sample is a hit (or it has none), else 0 */
    int32_t* hot_ids;       /* [B] ids of hot samples, ascending; first n_hot entries valid */
    int32_t* normal_ids;    /* [B] ids of the other samples, ascending; first n_normal entries valid */
    int32_t* n_hot_normal;  /* [2] = {n_hot, n_normal}; n_hot + n_normal = B */
} scars_classify_out;

/* Lifecycle.  scars_create copies the descriptor (not the tables); scars_destroy frees only the handle. */
int32_t scars_create(const scars_config* cfg, scars_handle** out);
int32_t scars_destroy(scars_handle* h);

/* Sizes of the buffers to allocate for a byte budget (Section IV: 128 MB .. 1024 MB caches; the budget
 * counts embedding weights only) and for batches of at most max_L lookups in max_G bags.  HOST only. */
int32_t scars_query_sizes(const scars_handle* h, int64_t budget_bytes, int64_t max_L, int64_t max_G,
                          scars_sizes* out);

/* Hand the allocated buffers to the handle.  Copies the table descriptors into the workspace and clears
 * the status word on `stream`; waits for that copy.  Forgets any previously built hot set: updated rows that are
 * only in the cache bound before are lost unless scars_flush_cache has written them back first. */
int32_t scars_bind_buffers(scars_handle* h, const scars_buffers* bufs, void* stream);

/* Skew table + top-k + cache fill (Section III: a frequency ranking over all rows, the hottest of which are kept on
 * the device; Section IV: fixed byte budget).
 *   counts[gid] += 1 for each of the Lp lookups of the profile batch (d_indices/d_offsets DEVICE,
 *   offsets has T*bags_per_table+1 entries);  then, unless accumulate == 2:
 *   k = min(N, floor(budget_bytes / R)); the hot set is the first k rows in the order (count descending,
 *   gid ascending); hot_gid[s] = s-th of them, slot_of[gid] = s or -1; cache[s] = the row's current value
 *   read from its pinned host table (and its Adagrad accumulator into state_cache[s]).
 *   accumulate: 0 = zero counts first; 1 = add to the existing counts, then select; 2 = add only.
 * If the cache holds rows updated since the last flush, they are written back first.
 * Lp = 0 with d_indices = NULL is allowed (select on the counts as they are).
 * Errors: INVALID_ARG, WORKSPACE (budget/Lp/bags beyond what was bound), cumulative lookups >= 2^32. */
int32_t scars_build_cache(scars_handle* h, const int32_t* d_indices, const int32_t* d_offsets, int64_t Lp,
                          int64_t bags_per_table, int64_t budget_bytes, int32_t accumulate, void* stream);

/* Rows actually cached by the last selecting scars_build_cache (HOST value, no device access); -1 if none. */
int64_t scars_cache_rows(const scars_handle* h);

/* Index -> cache-slot remap with ordered hit/miss compaction (the "lookup into the cached layer" that
 * Section IV finds to bound the forward pass).  Fills every array of `out`. */
int32_t scars_remap(scars_handle* h, const int32_t* d_indices, const int32_t* d_offsets, int64_t L, int64_t B,
                    const scars_remap_out* out, void* stream);

/* scars_remap for callers that cannot allocate device memory or hand over a workspace for this step (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the same outputs from the same kernels, but
 * the scratch this step needs (table descriptor, status word, per-tile hit and miss counts) lives in a 64 KiB static
 * device array inside the library, one copy per GPU, held until the process ends.  The call allocates nothing.
 * Limits: L <= SCARS_REMAP_STATIC_MAX_L (SCARS_ERR_WORKSPACE beyond), no unique_miss_gid (SCARS_ERR_INVALID_ARG).
 * It does not write the backward pass's pairs and starts no preparation (SCARS_TUNE_PAIRS_IN_REMAP / _PRESORT do
 * not apply).  Device-detected errors of this call are latched in the array's own status word, which
 * scars_sync_status reads and clears as well.  Every call on a GPU, from any handle, shares that GPU's array: calls
 * that overlap in time on one GPU (two streams, two handles) race on it and give unspecified hit/miss lists; calls in
 * stream order are safe, nothing in the array has to survive from one call to the next. */
#define SCARS_REMAP_STATIC_MAX_L (1 << 23)
int32_t scars_remap_static(scars_handle* h, const int32_t* d_indices, const int32_t* d_offsets, int64_t L, int64_t B,
                           const scars_remap_out* out, void* stream);

/* Pooled gather-sum (Fig. 1 step 2 with sum pooling; Section II-B for the cached rows):
 * d_out[g][:] = sum over the bag's lookups of the row, fp32, empty bag -> 0.  Hits are read from the HBM
 * cache; misses are first fetched from the pinned host tables into the workspace's staging area (the
 * only traffic on the host link) and read from there.  The sum runs in position order whatever the
 * source, so the result does not depend on the budget.  `rm` must come from scars_remap on this batch. */
int32_t scars_embedding_bag_fwd(scars_handle* h, const int32_t* d_indices, const int32_t* d_offsets, int64_t L,
                                int64_t B, const scars_remap_out* rm, float* d_out, void* stream);

/* Backward sorted-segment scatter-add with the row update (Section IV: backward + optimization stages):
 * lookups are ordered by (gid, position); each run of one gid sums d_grad_out[bag][:] (fp32 [T*B][D]) into
 * dW, then  SGD: w -= lr*dW   |   Adagrad: G += dW^2, w -= lr*dW/(sqrt(G)+eps)  (element-wise).
 * Cached rows are updated in the HBM cache (the host copy is stale until scars_flush_cache); other rows
 * are updated in place in pinned host memory.  bf16 rows are rounded to nearest even on store.
 * `out` may be NULL; otherwise the sorted segments are also written there. */
int32_t scars_embedding_bag_bwd_update(scars_handle* h, const int32_t* d_indices, const int32_t* d_offsets,
                                       int64_t L, int64_t B, const scars_remap_out* rm, const float* d_grad_out,
                                       float lr, float eps, const scars_bwd_out* out, void* stream);

/* The same update, and while it runs the missed rows of the NEXT batch are fetched over the host link (Fig. 1: the
 * transfer of a batch's embeddings; Section IV attributes the update's time to writes of rows to host memory, which
 * use the link's other direction).  For training loops that know the next batch:
 *     scars_remap(next) -> scars_embedding_bag_bwd_update_ahead(this, next_rm) -> scars_embedding_bag_fwd(next) -> ...
 * `next_rm`, `d_next_offsets`, `next_L`, `next_B`: the next batch as given to, and the outputs of, a scars_remap
 * already enqueued on `stream` (arrays of their own, without unique_miss_gid).  A missed row of the next batch is fetched now, into a second staging area and on a
 * stream the library owns, unless this update writes that row (a search in this batch's sorted list of distinct
 * rows); scars_embedding_bag_fwd for `next_rm` then fetches only the rows left out, after the update.  No row is read
 * while it may be written, so every result equals that of the calls made one batch after the other.  Under
 * SCARS_TUNE_PRESORT the integer half of the next batch's backward pass is prepared beside this update as well (in a
 * second set of workspace arrays), so that the next update starts at its reduce kernels.
 * Needs SCARS_TUNE_LOOKAHEAD = 1 (SCARS_ERR_INVALID_ARG otherwise).  Nothing is fetched ahead when L = 0. */
int32_t scars_embedding_bag_bwd_update_ahead(scars_handle* h, const int32_t* d_indices, const int32_t* d_offsets,
                                             int64_t L, int64_t B, const scars_remap_out* rm, const float* d_grad_out,
                                             float lr, float eps, const scars_bwd_out* out,
                                             const scars_remap_out* next_rm, const int32_t* d_next_offsets,
                                             int64_t next_L, int64_t next_B, void* stream);

/* Hot / normal samples (Section III: samples whose lookups are all cached versus the rest, so that mini-batches of
 * one kind can be composed).  Sample b is hot when none of its lookups over all T tables is a
 * miss; invalid lookups are ignored.  `rm` must come from scars_remap on this batch. */
int32_t scars_classify_samples(scars_handle* h, const int32_t* d_offsets, int64_t L, int64_t B, const scars_remap_out* rm,
                               const scars_classify_out* out, void* stream);

/* Sub-batch of selected samples (Section III: hot and normal samples are trained in separate mini-batches).  d_ids
 * (DEVICE int32, ascending sample numbers below B, e.g. hot_ids or normal_ids of scars_classify_samples) and *d_n
 * (DEVICE int32: how many of them, e.g. &n_hot_normal[0]) select the samples; the sub-batch keeps the table-major
 * layout with n samples per table: its bag t*n + j is bag t*B + d_ids[j] of the batch, lookups in their original
 * order, so its pooled sums are the selected rows of the batch's, bit for bit.  n stays on the device: read
 * n_lookups_bags back (or n_hot_normal) to call the per-batch entry points on the sub-batch with B = n. */
typedef struct {
    int32_t* indices;         /* DEVICE int32 [L]: first n_lookups entries valid */
    int32_t* offsets;         /* DEVICE int32 [T*B + 1]: first T*n + 1 entries valid */
    int32_t* n_lookups_bags;  /* DEVICE int32 [2] = {lookups, bags = T*n} of the sub-batch */
} scars_subbatch_out;
int32_t scars_partition_batch(scars_handle* h, const int32_t* d_indices, const int32_t* d_offsets, int64_t L, int64_t B,
                              const int32_t* d_ids, const int32_t* d_n, const scars_subbatch_out* out, void* stream);

/* Use of the cache by portion (the measurement of Fig. 4 in Section IV: samples of a mini-batch that touch each
 * successive part of the hotness-ordered cache).  d_usage[p], DEVICE int32 [n_portions] with n_portions <= 64,
 * receives the number of samples having at least one lookup whose slot lies in
 * [p * portion_rows, (p + 1) * portion_rows).  `rm` must come from scars_remap on this batch. */
int32_t scars_portion_usage(scars_handle* h, const int32_t* d_offsets, int64_t L, int64_t B, const scars_remap_out* rm,
                            int64_t portion_rows, int32_t n_portions, int32_t* d_usage, void* stream);

/* Budget chooser from the paper's expected-communication model (Section II-B).  With P(e) estimated from the
 * skew table as min(1, counts[e] / profile_samples), C = the first k rows of the ranking, d = dim and the batch
 * size tied to the cache by eq. (7), b = (M - k d) / a, an epoch of Q samples communicates (eq. (6), summed
 * over the T features, in parameters)
 *     cost(k) = T Q + (Q / b) d sum_{e not in C} (1 - (1 - P(e))^b).
 * Both calls BLOCK (one small kernel builds the rows-per-count table, the rest is host arithmetic). */
typedef struct {
    double device_params;      /* M: parameters that fit on the device */
    double per_sample_params;  /* a: parameters (weights share + activations) one sample of the batch needs */
    double samples_per_epoch;  /* Q */
    int64_t profile_samples;   /* samples behind the counts now in the skew table */
} scars_plan_in;

typedef struct {
    int64_t best_k;            /* rows to cache: the k with the smallest cost among those examined */
    double best_cost, best_batch;
    double cost_no_cache, batch_no_cache;   /* k = 0: coalescing only, eq. (5) */
    int64_t k_max;             /* largest k that still leaves room for one sample (b >= 1) */
} scars_plan_out;

/* cost(k) and its batch size for one k; INVALID_ARG if b < 1. */
int32_t scars_epoch_cost(scars_handle* h, const scars_plan_in* in, int64_t k, double* cost, double* batch, void* stream);

/* The paper's test for caching one more embedding (eq. (8)-(12)): with the first k rows of the ranking cached and e'
 * the next one, b = (M - k d) / a, b' = b - d / a, communication per epoch falls iff
 *     *lhs = 1 - (1 - P(e'))^b  >=  *t1 = sum_{e not in C'} (b (1 - (1 - P(e))^b') - b' (1 - (1 - P(e))^b)) / b'.
 * INVALID_ARG if k >= N or b' < 1.  BLOCKS like the other two. */
int32_t scars_caching_gain(scars_handle* h, const scars_plan_in* in, int64_t k, double* lhs, double* t1, void* stream);

/* Search over k in [0, k_max]: every k when k_max <= 4096, otherwise count-class borders and a narrowing grid. */
int32_t scars_plan_cache(scars_handle* h, const scars_plan_in* in, scars_plan_out* out, void* stream);

/* Write every cached row (and Adagrad accumulator) back to its pinned host table. */
int32_t scars_flush_cache(scars_handle* h, void* stream);

/* BLOCKS until `stream` is idle; returns the latched device-side error (then clears it) or SCARS_OK. */
int32_t scars_sync_status(scars_handle* h, void* stream);

/* Text of the last error on this handle (valid until the next call on it). */
const char* scars_last_error(const scars_handle* h);

/* Plumbing for callers without a HIP binding of their own: pinned host memory and a timed device-to-host /
 * host-to-device copy.  scars_host_alloc uses hipHostMalloc (device-mapped, coherent). */
int32_t scars_host_alloc(int64_t bytes, void** out);
int32_t scars_host_free(void* p);
int32_t scars_memcpy(void* dst, const void* src, int64_t bytes, int32_t kind /* 1 = H2D, 2 = D2H, 3 = D2D */,
                     void* stream);

/* Measurement aid: a plain streaming copy kernel (k_calib_copy; four 16-byte loads in flight per lane) of `bytes`
 * (multiple of 16) between two DEVICE buffers, used to scale hardware byte counters against a transfer of known size
 * and as the box's own copy rate. */
int32_t scars_calibration_copy(void* d_dst, const void* d_src, int64_t bytes, void* stream);

/* Measurement aid: a plain grid-stride read-only kernel over `bytes` (multiple of 16) of a DEVICE buffer; each
 * thread folds what it read into one 32-bit word of `d_sink` (DEVICE, at least SCARS_CALIB_SINK_BYTES).  Gives the
 * box's streaming read rate, the practical ceiling of a gather. */
#define SCARS_CALIB_SINK_BYTES (4 << 20)
int32_t scars_calibration_read(const void* d_src, int64_t bytes, void* d_sink, void* stream);

/* Measurement aid for the host link: n_granules pieces of granule_bytes (16 .. 1024, a power of two) move between
 * h_pinned (PINNED, host_bytes long) and d_buf (DEVICE, at least n_granules * granule_bytes), 16 bytes per lane and
 * granule_bytes / 16 lanes per piece, four pieces in flight per lane group, `workgroups` workgroups of 256 lanes.
 * Piece j of d_buf pairs with a piece of the host buffer picked by a hash of j (scattered != 0: the pattern in which
 * the rows of a batch lie in their tables) or with piece j modulo the host buffer (sequential).  to_host 0 reads the
 * host (the missed-row fetch of Fig. 1), 1 writes it (the cold-row update of Section IV).  Timed by the caller; gives
 * the link's ceiling for this access pattern, which below 256 bytes per piece is a request rate, not a byte rate. */
int32_t scars_calibration_link(void* h_pinned, int64_t host_bytes, void* d_buf, int64_t n_granules, int32_t granule_bytes,
                               int32_t scattered, int32_t to_host, int32_t workgroups, void* stream);

/* Per-kernel timing for measurement: when enabled, every kernel launch is bracketed by HIP events on the
 * caller's stream.  scars_profile_read waits for the stream, then returns up to `cap` records
 * (name pointer valid for the library's lifetime, launches, total milliseconds) and clears them. */
typedef struct {
    const char* name;
    int64_t launches;
    double total_ms;
} scars_kernel_time;
int32_t scars_profile_enable(scars_handle* h, int32_t on);
int32_t scars_profile_read(scars_handle* h, void* stream, scars_kernel_time* out, int32_t cap, int32_t* n_out);

#ifdef __cplusplus
}
#endif
#endif
