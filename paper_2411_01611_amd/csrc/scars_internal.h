// Internal host-side declarations shared by the translation units of libscars (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <initializer_list>
#include <map>
#include <string>
#include <vector>

#include "scars.h"

namespace scars {

constexpr int kBlock = 256;          // threads per workgroup everywhere: 4 wave64
constexpr int kWave = 64;
constexpr int kScanTile = 2048;      // items per workgroup in the ordered-compaction kernels
constexpr int kSortRoundsSmall = 4;   // radix-sort tile = 256 * rounds pairs: 1024 for inputs up to 2^18 pairs,
constexpr int kSortRoundsMid = 8;     // 2048 below 2^22,
constexpr int kSortRoundsLarge = 16;   // 4096 from there on
constexpr int kSortMaxBins = 512;     // up to 9 bits per pass
constexpr int kSmallSortCap = 4096;   // pairs per table the one-workgroup-per-table sort takes
constexpr int kSelBins = 2048;       // radix-select bins per pass (11 + 11 + 10 bits)
constexpr int kPlanBins = 65536;      // count-of-counts bins of the budget chooser; larger counts go to a short list
constexpr int kPlanBigCap = 4096;
constexpr int64_t kSegViaLocMaxL = 1 << 20;   // up to this many lookups a run's slot is taken from remap's per-lookup arrays
constexpr int kLongRunMin = 64;      // runs longer than this are cut into tasks of this many lookups
constexpr int64_t kStaticRemapMaxL = SCARS_REMAP_STATIC_MAX_L;   // largest batch of scars_remap_static

inline int64_t align_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }
inline int64_t div_up(int64_t x, int64_t a) { return (x + a - 1) / a; }

// Device-resident table descriptors (lives at the start of the workspace).
struct Meta {
    const void* table[SCARS_MAX_TABLES];   // pinned host row storage
    float* state[SCARS_MAX_TABLES];        // pinned host Adagrad accumulators (or null)
    int32_t row_base[SCARS_MAX_TABLES + 1];
    int32_t num_tables;
    int32_t pad[3];
};

// Everything carved out of the caller's workspace blob.
struct Workspace {
    Meta* meta;
    int32_t* status;          // [4] latched device-side error word
    // selection (build_cache)
    uint32_t* sel_hist;       // [3][kSelBins]
    uint32_t* sel_state;      // [8]: prefix, k_rem, (pad)
    uint32_t* blk_gt;         // [nbN + 1]
    uint32_t* blk_eq;         // [nbN + 1]
    uint32_t* win_key[2];     // [k] double buffer
    int32_t* win_gid[2];      // [k]
    // per batch
    uint32_t* blk_hit;        // [tiles of max(max_L, max_G) + 1] per-tile counts of the ordered compactions
    uint32_t* blk_miss;       // same
    uint32_t* sort_hist;      // [nbS * bins] per-tile digit histogram (a row per tile), nbS tiles for max(max_L, k) pairs
    uint32_t* sort_tot;       // [kSortMaxBins]
    uint32_t* key_buf[2];     // [max_L]
    uint32_t* val_buf[2];     // [max_L]
    int32_t* seg_start;       // [max_L + 1] (used when the caller passes no bwd_out)
    int32_t* unique_gid;      // [max_L]
    int32_t* n_unique;        // [2]
    int32_t* unique_slot;     // [max_L] cache slot (or -1) of each distinct row of the batch
    uint32_t* first_bag;      // [max_L] bag of the first lookup of each distinct row
    double* partial;          // [chunks][2][D] fp64 partial sums of long runs, chunks of kLongRunMin sorted positions
    int32_t* chunk_run;       // [chunks + 1] run (segment) index that holds each chunk's first position
    uint32_t* blk_seg_a;      // [tiles+1] x2: tile counters of the backward pass's run-start compaction (its own pair:
    uint32_t* blk_seg_b;      //   that half of the pass may run on the side stream beside calls that use blk_hit/blk_miss)
    uint32_t* plan_cc;        // [kPlanBins] rows per count value, [kPlanBigCap] counts at or above kPlanBins, [4] their number
    void* staging[2];         // [max_L][R] rows fetched over the host link; the second area is for rows fetched ahead
    // a second set of the arrays that hold a batch's sorted pairs and run starts, so that the next batch's can be
    // prepared while this batch's are still being read (look-ahead); swap_segment_sets exchanges the two
    struct SegSet {
        uint32_t* key_buf[2];
        uint32_t* val_buf[2];
        int32_t* seg_start;
        int32_t* unique_gid;
        int32_t* n_unique;
        int32_t* unique_slot;
        uint32_t* first_bag;
        int32_t* chunk_run;
    } alt;
    uint8_t* fetched;         // [max_L] 1 = this missed lookup's row was fetched ahead
    int64_t total_bytes;
};

struct KernelTimer {
    struct Rec { const char* name; hipEvent_t a, b; int64_t tag; };
    std::vector<Rec> pending;
};

}  // namespace scars

struct scars_handle {
    // descriptor
    int32_t T = 0, D = 0, dtype = 0, optimizer = 0;
    int64_t N = 0;
    int32_t R = 0;                       // row bytes
    std::vector<int64_t> rows;
    std::vector<int64_t> row_base;       // [T+1]
    std::vector<void*> host_tables;
    std::vector<float*> host_state;
    // bound buffers
    bool bound = false;
    scars_buffers buf{};
    int64_t k_cap = 0;
    scars::Workspace ws{};
    // state
    bool built = false;
    bool dirty = false;                  // cache holds rows newer than the host tables
    int64_t k = -1;
    uint64_t profiled = 0;               // cumulative lookups histogrammed
    // staging areas: area a holds the missed rows of the batch whose remap wrote stg[a].loc
    struct Staged { bool valid = false; const int32_t* loc = nullptr; } stg[2];
    int staged_area(const int32_t* loc) const {
        for (int a = 0; a < 2; ++a) if (stg[a].valid && stg[a].loc == loc) return a;
        return -1;
    }
    // look-ahead (SCARS_TUNE_LOOKAHEAD): rows of the next batch fetched while this batch is updated
    bool lookahead = false;
    struct { bool valid = false; const int32_t* loc = nullptr; const int32_t* miss_gid = nullptr; int area = 0; } ahead;   // what was fetched ahead, where
    hipEvent_t ev_pf_fork = nullptr, ev_pf_done = nullptr;
    bool pf_pending = false;             // a fetch on pool_stream that no other stream has waited for yet
    bool ahead_active = false;           // the backward pass being enqueued has a fetch running beside it
    std::string err;
    // side stream: the integer half of the backward pass can be started by remap and run beside the forward pass
    hipStream_t side = nullptr;
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    hipStream_t pool_stream = nullptr;   // forward pass: bags that need no fetched row, pooled beside the fetch
    hipEvent_t ev_pool_fork = nullptr, ev_pool_join = nullptr;
    bool side_pending = false;           // ev_join has been recorded and no stream has been made to wait for it yet
    bool presort_valid = false;          // the workspace holds the segments of the batch described below
    const int32_t *presort_gid = nullptr, *presort_loc = nullptr, *presort_off = nullptr;
    int64_t presort_L = 0, presort_B = 0;
    bool presort_staged = false;
    int presort_res = 0;
    // (gid, bag) pairs of the batch described below are in the first sort buffer (written by scars_remap)
    bool pairs_valid = false;
    const int32_t* pairs_gid = nullptr;
    const int32_t* pairs_off = nullptr;
    int64_t pairs_L = 0, pairs_B = 0;
    int64_t n_ahead_used = 0;            // forward passes that used rows fetched ahead
    int64_t n_ahead_timed = 0;           // updates with a fetch on the library's stream beside them, timed in profile mode
    int64_t n_ahead_serial = 0;          // ... of which the fetch and the update did not run at the same time
    int64_t timer_tag = 0;               // > 0: launches being enqueued belong to the update/fetch pair with this number
    int64_t timer_serial = 0;
    bool fused_fetch = true;             // the fetch ahead rides in the update's launch when it can
    int64_t n_prepared_used = 0;         // bwd_update calls that used segments prepared on the side stream
    // launch tuning (scars_set_tuning)
    int64_t presort_min_L = 0;           // > 0: remap starts the backward pass's sort on the side stream for batches this large
    int64_t update_max_blocks = 0;       // workgroups of the per-row update kernel (it strides over the rows); 0 = by case
    bool pairs_in_remap = true;          // scars_remap also writes the backward pass's (gid, bag) pairs
    int64_t table_lookups_limit = 0;     // > 0: the caller states that no table gets more lookups than this in a batch
    // the forward pass of this batch has already sorted each table's pairs (in the launch that fetches the missed rows):
    int64_t n_small_sorted_used = 0;     // backward passes that found their pieces sorted by the forward pass
    bool small_sorted = false;
    bool small_runs = false;             // ... and left each run's length and row source for an update by position,
    bool small_runs_staged = false;      //     with cold rows read from the staging area that forward pass filled
    const int32_t *small_gid = nullptr, *small_off = nullptr;
    int64_t small_L = 0, small_B = 0;
    // whether the per-table sort applies to this handle at all
    bool small_sort_applies() const { return table_lookups_limit > 0 && table_lookups_limit <= scars::kSmallSortCap && 2 * T <= scars::kSortMaxBins; }
    int fused_scan_max_tiles = 4096;     // compaction: up to this many tiles the writer sums the tile counts itself
    int64_t fused_long_max_L = ((int64_t)1 << 31) - 1;   // backward: up to this many lookups long runs and rows share one launch
    // per-kernel timing
    bool profile = false;
    scars::KernelTimer timer;
};

namespace scars {

int32_t fail(scars_handle* h, int32_t code, const std::string& msg);
// scars_api.hip: make the library's side stream wait for everything enqueued on s so far
hipError_t side_fork(scars_handle* h, hipStream_t s);
int32_t hip_fail(scars_handle* h, hipError_t e, const char* what);

// RAII bracket that records a start/stop event pair around one kernel launch when profiling is on.
struct Timed {
    scars_handle* h;
    hipStream_t s;
    const char* name;
    hipEvent_t a = nullptr, b = nullptr;
    int64_t tag = 0;
    Timed(scars_handle* h_, hipStream_t s_, const char* n);
    ~Timed();
};

Workspace carve(const scars_handle* h, void* base, int64_t k_cap, int64_t max_L, int64_t max_G);

// ---- launchers (each enqueues on `s`; returns hipGetLastError) -------------------------------------
// k_sort.hip
hipError_t launch_radix_sort_pairs(scars_handle* h, hipStream_t s, uint32_t* key[2], uint32_t* val[2], int64_t n,
                                   const int32_t* d_n /*device-side pair count bounded by n, or null*/, int bits,
                                   int* result_buffer /*0 or 1: which buffer holds the result*/);
// k_sort.hip: for a batch whose tables each hold at most `limit` (<= kSmallSortCap) of the L pairs (positions
// [off[t*B], off[(t+1)*B]) belong to table t): one workgroup per table sorts its piece in LDS, from key[0] / val[0]
// into the same positions of key[1] / val[1]; per-table counts go to ws.sort_hist (valid pairs [T], distinct rows [T])
// `run` (may be null): also write each run's length and row source at its first position (see SmallRunArgs)
struct SmallRunArgs;
hipError_t launch_small_sort(scars_handle* h, hipStream_t s, uint32_t* key[2], uint32_t* val[2], const int32_t* off,
                             int64_t L, int64_t B, const SmallRunArgs* run);
// k_build_cache.hip
hipError_t launch_fill_u32(scars_handle* h, hipStream_t s, uint32_t* p, int64_t n, uint32_t v);
hipError_t launch_histogram(scars_handle* h, hipStream_t s, const int32_t* idx, const int32_t* off, int64_t L,
                            int64_t B);
hipError_t launch_select_and_fill(scars_handle* h, hipStream_t s, int64_t k);
hipError_t launch_flush(scars_handle* h, hipStream_t s);
hipError_t launch_calib_copy(hipStream_t s, void* dst, const void* src, int64_t bytes);
hipError_t launch_calib_read(hipStream_t s, const void* src, int64_t bytes, void* sink);
hipError_t launch_calib_link(hipStream_t s, void* host, int64_t host_bytes, void* dev, int64_t n, int granule_bytes,
                             int scattered, int to_host, int blocks);
// k_remap.hip
hipError_t launch_remap(scars_handle* h, hipStream_t s, const int32_t* idx, const int32_t* off, int64_t L, int64_t B,
                        const scars_remap_out* out);
// k_remap.hip: the same three launches with the library's static device array in place of the workspace
hipError_t launch_remap_static(scars_handle* h, hipStream_t s, const int32_t* idx, const int32_t* off, int64_t L, int64_t B,
                               const scars_remap_out* out);
// k_remap.hip: the status word inside that array on the current device, or null if nothing has used the array there
int32_t* static_status_if_used();
// k_remap.hip (also used by k_classify.hip): exclusive scan of two per-tile count arrays, totals to out2[0..1]
__global__ void k_remap_scan(uint32_t* a, uint32_t* b, int n, int32_t* out2);
// k_classify.hip
hipError_t launch_classify(scars_handle* h, hipStream_t s, const int32_t* off, int64_t L, int64_t B,
                           const scars_remap_out* rm, const scars_classify_out* out);
hipError_t launch_portion_usage(scars_handle* h, hipStream_t s, const int32_t* off, int64_t L, int64_t B,
                                const scars_remap_out* rm, int64_t portion_rows, int32_t n_portions, int32_t* usage);
hipError_t launch_partition(scars_handle* h, hipStream_t s, const int32_t* idx, const int32_t* off, int64_t L, int64_t B,
                            const int32_t* ids, const int32_t* d_n, const scars_subbatch_out* out);
// k_plan.hip
hipError_t launch_count_of_counts(scars_handle* h, hipStream_t s);
double plan_cost(const std::vector<std::pair<uint32_t, int64_t>>& classes, int T, int64_t n_samples, int64_t k, double M,
                 double a, double d, double Q, double* b_out);
// k_fwd.hip
hipError_t launch_fwd(scars_handle* h, hipStream_t s, const int32_t* off, int64_t L, int64_t B,
                      const scars_remap_out* rm, float* out);
// k_bwd.hip
hipError_t launch_bwd(scars_handle* h, hipStream_t s, const int32_t* off, int64_t L, int64_t B,
                      const scars_remap_out* rm, const float* grad, float lr, float eps, const scars_bwd_out* out,
                      const scars_remap_out* next_rm, const int32_t* next_off, int64_t next_L, int64_t next_B);
// k_fwd.hip: missed rows of a remapped batch that are not in the sorted list `excl` -> staging area `area`
// (`fused` set: only flags the rows and describes the job in *fused / *fused_blocks, for the caller's own launch)
struct StageArgs;
hipError_t launch_fetch_ahead(scars_handle* h, hipStream_t s, const scars_remap_out* next_rm, int64_t next_L,
                              const int32_t* excl, const int32_t* n_excl, int area, StageArgs* fused, int* fused_blocks);
hipError_t ensure_pool_stream(scars_handle* h);
hipError_t pf_join(scars_handle* h, hipStream_t s);
void swap_segment_sets(scars_handle* h);
hipError_t start_presort(scars_handle* h, hipStream_t s, const int32_t* off, int64_t L, int64_t B, const scars_remap_out* rm);
hipError_t launch_bwd_segments(scars_handle* h, hipStream_t s, const int32_t* off, int64_t L, int64_t B,
                               const scars_remap_out* rm, bool staged, const scars_bwd_out* out, int* res_out,
                               bool* by_position /*null: the list of runs is wanted; else set when the per-table sort
                                                   has left the runs by position instead (k_small_update)*/);

}  // namespace scars
