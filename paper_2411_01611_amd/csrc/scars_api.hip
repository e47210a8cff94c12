// C ABI of libscars: handle lifecycle, buffer binding, argument checks, and the four entry points.
// Every device step is a kernel in the k_*.hip files; this file only validates and enqueues.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <functional>

#include "scars_internal.h"

using namespace scars;

namespace scars {

int32_t fail(scars_handle* h, int32_t code, const std::string& msg) {
    if (h) h->err = msg;
    return code;
}

int32_t hip_fail(scars_handle* h, hipError_t e, const char* what) {
    return fail(h, SCARS_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

Timed::Timed(scars_handle* h_, hipStream_t s_, const char* n) : h(h_), s(s_), name(n) {
    if (h && h->profile) {
        tag = h->timer_tag;
        if (hipEventCreate(&a) == hipSuccess && hipEventCreate(&b) == hipSuccess) {
            (void)hipEventRecord(a, s);
        } else {
            a = b = nullptr;
        }
    }
}

Timed::~Timed() {
    if (a && b) {
        (void)hipEventRecord(b, s);
        h->timer.pending.push_back({name, a, b, tag});
    }
}

// Lay the scratch arrays out in the caller's workspace blob.  With base == nullptr only sizes are computed.
Workspace carve(const scars_handle* h, void* base, int64_t k_cap, int64_t max_L, int64_t max_G) {
    Workspace w{};
    int64_t off = 0;
    auto take = [&](int64_t bytes) -> void* {
        void* p = base ? (char*)base + off : nullptr;
        off += align_up(std::max<int64_t>(bytes, 16), 256);
        return p;
    };
    const int64_t nbN = div_up(h->N, kScanTile), nbL = std::max<int64_t>(1, div_up(max_L, kScanTile));
    const int64_t nbS = std::max<int64_t>(1, div_up(std::max(max_L, k_cap), kBlock * kSortRoundsSmall));
    w.meta = (Meta*)take(sizeof(Meta));
    w.status = (int32_t*)take(16);
    w.sel_hist = (uint32_t*)take(3 * kSelBins * 4);
    w.sel_state = (uint32_t*)take(32);
    w.blk_gt = (uint32_t*)take((nbN + 1) * 4);
    w.blk_eq = (uint32_t*)take((nbN + 1) * 4);
    for (int i = 0; i < 2; ++i) {
        w.win_key[i] = (uint32_t*)take(k_cap * 4);
        w.win_gid[i] = (int32_t*)take(k_cap * 4);
    }
    const int64_t nbLG = std::max<int64_t>(nbL, div_up(max_G, kScanTile));
    w.blk_hit = (uint32_t*)take((nbLG + 1) * 4);
    w.blk_miss = (uint32_t*)take((nbLG + 1) * 4);
    w.sort_hist = (uint32_t*)take(kSortMaxBins * nbS * 4);
    w.sort_tot = (uint32_t*)take(kSortMaxBins * 4);
    for (int i = 0; i < 2; ++i) {
        w.key_buf[i] = (uint32_t*)take(max_L * 4);
        w.val_buf[i] = (uint32_t*)take(max_L * 4);
    }
    w.seg_start = (int32_t*)take((max_L + 1) * 4);
    w.unique_gid = (int32_t*)take(max_L * 4);
    w.n_unique = (int32_t*)take(16);
    w.unique_slot = (int32_t*)take(max_L * 4);
    w.first_bag = (uint32_t*)take(max_L * 4);
    const int64_t chunks = nbL * (kScanTile / kLongRunMin);    // whole scan tiles: the counters are cleared per tile
    w.partial = (double*)take(chunks * 2 * h->D * 8);
    w.chunk_run = (int32_t*)take((chunks + 1) * 4);
    w.blk_seg_a = (uint32_t*)take((nbLG + 1) * 4);
    w.blk_seg_b = (uint32_t*)take((nbLG + 1) * 4);
    w.plan_cc = (uint32_t*)take((kPlanBins + kPlanBigCap + 4) * 4);
    w.staging[0] = take(max_L * h->R);
    w.staging[1] = take(max_L * h->R);
    w.fetched = (uint8_t*)take(max_L);
    for (int i = 0; i < 2; ++i) {
        w.alt.key_buf[i] = (uint32_t*)take(max_L * 4);
        w.alt.val_buf[i] = (uint32_t*)take(max_L * 4);
    }
    w.alt.seg_start = (int32_t*)take((max_L + 1) * 4);
    w.alt.unique_gid = (int32_t*)take(max_L * 4);
    w.alt.n_unique = (int32_t*)take(16);
    w.alt.unique_slot = (int32_t*)take(max_L * 4);
    w.alt.first_bag = (uint32_t*)take(max_L * 4);
    w.alt.chunk_run = (int32_t*)take((chunks + 1) * 4);
    w.total_bytes = off;
    return w;
}

// Make stream s wait for work enqueued on the side stream, if any is outstanding.
static hipError_t side_join(scars_handle* h, hipStream_t s) {
    if (!h->side_pending) return hipSuccess;
    h->side_pending = false;
    return hipStreamWaitEvent(s, h->ev_join, 0);
}

static hipError_t ensure_side_stream(scars_handle* h) {
    hipError_t e = hipSuccess;
    if (!h->side && (e = hipStreamCreateWithFlags(&h->side, hipStreamNonBlocking)) != hipSuccess) return e;
    if (!h->ev_fork && (e = hipEventCreateWithFlags(&h->ev_fork, hipEventDisableTiming)) != hipSuccess) return e;
    if (!h->ev_join && (e = hipEventCreateWithFlags(&h->ev_join, hipEventDisableTiming)) != hipSuccess) return e;
    return e;
}

// Make the side stream (default priority; created when buffers are first bound) wait for everything enqueued on s so far.
hipError_t side_fork(scars_handle* h, hipStream_t s) {
    hipError_t e = ensure_side_stream(h);
    if (e != hipSuccess) return e;
    if ((e = hipEventRecord(h->ev_fork, s)) != hipSuccess) return e;
    return hipStreamWaitEvent(h->side, h->ev_fork, 0);
}

void swap_segment_sets(scars_handle* h) {
    Workspace& w = h->ws;
    for (int i = 0; i < 2; ++i) {
        std::swap(w.key_buf[i], w.alt.key_buf[i]);
        std::swap(w.val_buf[i], w.alt.val_buf[i]);
    }
    std::swap(w.seg_start, w.alt.seg_start);
    std::swap(w.unique_gid, w.alt.unique_gid);
    std::swap(w.n_unique, w.alt.n_unique);
    std::swap(w.unique_slot, w.alt.unique_slot);
    std::swap(w.first_bag, w.alt.first_bag);
    std::swap(w.chunk_run, w.alt.chunk_run);
}

// Make stream s wait for rows being fetched ahead on the library's third stream, if any are outstanding.
hipError_t pf_join(scars_handle* h, hipStream_t s) {
    if (!h->pf_pending) return hipSuccess;
    h->pf_pending = false;
    return hipStreamWaitEvent(s, h->ev_pf_done, 0);
}

// The integer half of the backward pass of a remapped batch (pairs, sort, run starts), started on the side stream
// behind everything enqueued on s so far; scars_embedding_bag_bwd_update joins it when it is called for that batch.
hipError_t start_presort(scars_handle* h, hipStream_t s, const int32_t* off, int64_t L, int64_t B, const scars_remap_out* rm) {
    hipError_t e = side_fork(h, s);
    if (e != hipSuccess) return e;
    const bool staged = h->k < h->N;   // misses are possible: the forward pass stages them
    e = launch_bwd_segments(h, h->side, off, L, B, rm, staged, nullptr, &h->presort_res, nullptr);
    if (e == hipSuccess) e = hipEventRecord(h->ev_join, h->side);
    if (e != hipSuccess) return e;
    h->side_pending = true;
    h->presort_valid = true;
    h->presort_gid = rm->gid; h->presort_loc = rm->loc; h->presort_off = off;
    h->presort_L = L; h->presort_B = B; h->presort_staged = staged;
    return hipSuccess;
}

static int64_t budget_rows(const scars_handle* h, int64_t budget_bytes) {
    if (budget_bytes <= 0) return 0;
    return std::min<int64_t>(h->N, budget_bytes / h->R);
}

}  // namespace scars

extern "C" {

int32_t scars_create(const scars_config* cfg, scars_handle** out) {
    if (!cfg || !out) return SCARS_ERR_INVALID_ARG;
    *out = nullptr;
    if (cfg->num_tables < 1 || cfg->num_tables > SCARS_MAX_TABLES || !cfg->rows || !cfg->host_tables || cfg->dim < 1)
        return SCARS_ERR_INVALID_ARG;
    if (cfg->dtype != SCARS_DTYPE_F32 && cfg->dtype != SCARS_DTYPE_BF16) return SCARS_ERR_INVALID_ARG;
    if (cfg->optimizer != SCARS_OPT_SGD && cfg->optimizer != SCARS_OPT_ADAGRAD) return SCARS_ERR_INVALID_ARG;
    if (cfg->optimizer == SCARS_OPT_ADAGRAD && !cfg->host_state) return SCARS_ERR_INVALID_ARG;
    const int64_t R = (int64_t)cfg->dim * (cfg->dtype == SCARS_DTYPE_F32 ? 4 : 2);
    if (R % 16 != 0 || R > SCARS_MAX_ROW_BYTES) return SCARS_ERR_INVALID_ARG;
    scars_handle* h = new (std::nothrow) scars_handle();
    if (!h) return SCARS_ERR_INVALID_ARG;
    h->T = cfg->num_tables; h->D = cfg->dim; h->dtype = cfg->dtype; h->optimizer = cfg->optimizer; h->R = (int32_t)R;
    h->row_base.push_back(0);
    for (int t = 0; t < h->T; ++t) {
        if (cfg->rows[t] < 1 || !cfg->host_tables[t] ||
            (cfg->optimizer == SCARS_OPT_ADAGRAD && !cfg->host_state[t])) { delete h; return SCARS_ERR_INVALID_ARG; }
        h->rows.push_back(cfg->rows[t]);
        h->N += cfg->rows[t];
        if (h->N >= ((int64_t)1 << 31)) { delete h; return SCARS_ERR_INVALID_ARG; }
        h->row_base.push_back(h->N);
        h->host_tables.push_back(cfg->host_tables[t]);
        h->host_state.push_back(cfg->optimizer == SCARS_OPT_ADAGRAD ? cfg->host_state[t] : nullptr);
    }
    *out = h;
    return SCARS_OK;
}

int32_t scars_set_tuning(scars_handle* h, int32_t which, int64_t value) {
    if (!h) return SCARS_ERR_INVALID_ARG;
    if (value < 0 || value >= ((int64_t)1 << 31)) return fail(h, SCARS_ERR_INVALID_ARG, "set_tuning: value out of range");
    switch (which) {
        case SCARS_TUNE_FUSED_SCAN_MAX_TILES: h->fused_scan_max_tiles = (int)std::min<int64_t>(value, 4096); break;
        case SCARS_TUNE_PRESORT: h->presort_min_L = value; break;
        case SCARS_TUNE_FUSED_LONG_MAX_L: h->fused_long_max_L = value; break;
        case SCARS_TUNE_PAIRS_IN_REMAP: h->pairs_in_remap = value != 0; break;
        case SCARS_TUNE_LOOKAHEAD: h->lookahead = value != 0; break;
        case SCARS_TUNE_UPDATE_MAX_BLOCKS: h->update_max_blocks = std::min<int64_t>(value, 1 << 16); break;
        case SCARS_TUNE_FUSED_FETCH: h->fused_fetch = value != 0; break;
        case SCARS_TUNE_MAX_TABLE_LOOKUPS: h->table_lookups_limit = value; break;
        default: return fail(h, SCARS_ERR_INVALID_ARG, "set_tuning: unknown parameter");
    }
    return SCARS_OK;
}

int64_t scars_get_counter(const scars_handle* h, int32_t which) {
    if (!h) return -1;
    switch (which) {
        case SCARS_COUNTER_PREPARED_USED: return h->n_prepared_used;
        case SCARS_COUNTER_AHEAD_USED: return h->n_ahead_used;
        case SCARS_COUNTER_AHEAD_TIMED: return h->n_ahead_timed;
        case SCARS_COUNTER_AHEAD_NOT_OVERLAPPED: return h->n_ahead_serial;
        case SCARS_COUNTER_SORTED_IN_FWD_USED: return h->n_small_sorted_used;
        default: return -1;
    }
}

int32_t scars_destroy(scars_handle* h) {
    if (!h) return SCARS_ERR_INVALID_ARG;
    if (h->pool_stream) {
        (void)hipStreamSynchronize(h->pool_stream);
        (void)hipStreamDestroy(h->pool_stream);
    }
    for (hipEvent_t ev : {h->ev_pool_fork, h->ev_pool_join, h->ev_pf_fork, h->ev_pf_done})
        if (ev) (void)hipEventDestroy(ev);
    if (h->side) {
        (void)hipStreamSynchronize(h->side);
        (void)hipStreamDestroy(h->side);
    }
    if (h->ev_fork) (void)hipEventDestroy(h->ev_fork);
    if (h->ev_join) (void)hipEventDestroy(h->ev_join);
    for (auto& p : h->timer.pending) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
    delete h;
    return SCARS_OK;
}

int32_t scars_query_sizes(const scars_handle* h, int64_t budget_bytes, int64_t max_L, int64_t max_G, scars_sizes* out) {
    if (!h || !out || budget_bytes < 0 || max_L < 0 || max_G < 0) return SCARS_ERR_INVALID_ARG;
    const int64_t k = budget_rows(h, budget_bytes);
    if (k + max_L >= ((int64_t)1 << 31) || max_G >= ((int64_t)1 << 31)) return SCARS_ERR_INVALID_ARG;
    auto a = [](int64_t b) { return align_up(std::max<int64_t>(b, 16), 256); };
    out->k = k;
    out->counts_bytes = a(h->N * 4);
    out->slot_of_bytes = a(h->N * 4);
    out->hot_gid_bytes = a(k * 4);
    out->cache_bytes = a(k * h->R);
    out->state_cache_bytes = h->optimizer == SCARS_OPT_ADAGRAD ? a(k * (int64_t)h->D * 4) : 0;
    out->workspace_bytes = carve(h, nullptr, k, max_L, max_G).total_bytes;
    out->per_lookup_bytes = a(max_L * 4);
    out->seg_start_bytes = a((max_L + 1) * 4);
    out->out_bytes = a(max_G * (int64_t)h->D * 4);
    return SCARS_OK;
}

int32_t scars_bind_buffers(scars_handle* h, const scars_buffers* b, void* stream) {
    if (!h) return SCARS_ERR_INVALID_ARG;
    if (!b || !b->counts || !b->slot_of || !b->workspace || b->budget_bytes < 0 || b->max_L < 0 || b->max_G < 0)
        return fail(h, SCARS_ERR_INVALID_ARG, "bind_buffers: null buffer or negative size");
    const int64_t k = budget_rows(h, b->budget_bytes);
    if (k + b->max_L >= ((int64_t)1 << 31)) return fail(h, SCARS_ERR_INVALID_ARG, "bind_buffers: k + max_L >= 2^31");
    if (k > 0 && (!b->hot_gid || !b->cache || (h->optimizer == SCARS_OPT_ADAGRAD && !b->state_cache)))
        return fail(h, SCARS_ERR_INVALID_ARG, "bind_buffers: cache buffers missing");
    {   // every buffer at least as large as scars_query_sizes says for these arguments
        scars_sizes need;
        if (scars_query_sizes(h, b->budget_bytes, b->max_L, b->max_G, &need) != SCARS_OK)
            return fail(h, SCARS_ERR_INVALID_ARG, "bind_buffers: sizes out of range");
        const bool adagrad = h->optimizer == SCARS_OPT_ADAGRAD;
        if (b->counts_bytes < need.counts_bytes || b->slot_of_bytes < need.slot_of_bytes ||
            b->workspace_bytes < need.workspace_bytes ||
            (k > 0 && (b->hot_gid_bytes < need.hot_gid_bytes || b->cache_bytes < need.cache_bytes ||
                       (adagrad && b->state_cache_bytes < need.state_cache_bytes))))
            return fail(h, SCARS_ERR_WORKSPACE, "bind_buffers: a buffer is smaller than scars_query_sizes asks for");
    }
    // The library's two streams are created here, not on first use: a process has few hardware queues, handed out as
    // streams are created, and a caller who binds before creating streams of its own keeps these two off its queue.
    {
        hipError_t es = ensure_side_stream(h);
        if (es == hipSuccess) es = ensure_pool_stream(h);
        if (es != hipSuccess) return hip_fail(h, es, "bind_buffers(streams)");
    }
    if (h->side) (void)hipStreamSynchronize(h->side);   // nothing may still be using the buffers bound before
    if (h->pool_stream) (void)hipStreamSynchronize(h->pool_stream);
    h->pf_pending = false;
    h->side_pending = false;
    h->presort_valid = false;
    h->pairs_valid = false;
    h->small_sorted = false;
    h->buf = *b;
    h->k_cap = k;
    h->ws = carve(h, b->workspace, k, b->max_L, b->max_G);
    h->bound = true; h->built = false; h->dirty = false; h->k = -1; h->profiled = 0;
    h->stg[0].valid = h->stg[1].valid = false; h->ahead.valid = false;
    Meta* m = new Meta();
    std::memset(m, 0, sizeof(Meta));
    for (int t = 0; t < h->T; ++t) {
        m->table[t] = h->host_tables[t];
        m->state[t] = h->host_state[t];
        m->row_base[t] = (int32_t)h->row_base[t];
    }
    m->row_base[h->T] = (int32_t)h->row_base[h->T];
    m->num_tables = h->T;
    hipStream_t s = (hipStream_t)stream;
    hipError_t e = hipMemcpyAsync(h->ws.meta, m, sizeof(Meta), hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = launch_fill_u32(h, s, (uint32_t*)h->ws.status, 4, 0u);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    delete m;
    if (e != hipSuccess) { h->bound = false; return hip_fail(h, e, "bind_buffers"); }
    return SCARS_OK;
}

static int32_t check_batch(scars_handle* h, const int32_t* idx, const int32_t* off, int64_t L, int64_t B, const char* who) {
    if (!h) return SCARS_ERR_INVALID_ARG;
    if (!h->bound) return fail(h, SCARS_ERR_WORKSPACE, std::string(who) + ": no buffers bound");
    if (!off || L < 0 || B < 0 || (L > 0 && !idx)) return fail(h, SCARS_ERR_INVALID_ARG, std::string(who) + ": null or negative argument");
    if (L > h->buf.max_L || (int64_t)h->T * B > h->buf.max_G)
        return fail(h, SCARS_ERR_WORKSPACE, std::string(who) + ": batch larger than the bound max_L / max_G");
    return SCARS_OK;
}

int32_t scars_build_cache(scars_handle* h, const int32_t* d_indices, const int32_t* d_offsets, int64_t Lp,
                          int64_t bags_per_table, int64_t budget_bytes, int32_t accumulate, void* stream) {
    if (!h) return SCARS_ERR_INVALID_ARG;
    if (!h->bound) return fail(h, SCARS_ERR_WORKSPACE, "build_cache: no buffers bound");
    if (accumulate < 0 || accumulate > 2 || budget_bytes < 0 || Lp < 0 || bags_per_table < 0)
        return fail(h, SCARS_ERR_INVALID_ARG, "build_cache: bad argument");
    const bool have_stream = Lp > 0 || d_offsets != nullptr;
    if (have_stream) {
        int32_t rc = check_batch(h, d_indices, d_offsets, Lp, bags_per_table, "build_cache");
        if (rc) return rc;
    }
    const int64_t k = budget_rows(h, budget_bytes);
    if (accumulate != 2 && k > h->k_cap) return fail(h, SCARS_ERR_WORKSPACE, "build_cache: budget above the bound budget");
    const uint64_t before = accumulate == 0 ? 0 : h->profiled;
    if (before + (uint64_t)Lp >= ((uint64_t)1 << 32))
        return fail(h, SCARS_ERR_INVALID_ARG, "build_cache: cumulative lookups >= 2^32 would overflow the uint32 counts");
    hipStream_t s = (hipStream_t)stream;
    hipError_t e = side_join(h, s);   // segments being prepared on the side stream read slot_of and the sort buffers
    if (e == hipSuccess) e = pf_join(h, s);
    if (e != hipSuccess) return hip_fail(h, e, "build_cache(join)");
    h->presort_valid = false;
    h->small_sorted = false;    // (the selection sorts in the same buffers)
    if (accumulate != 2 && h->built && h->dirty) {   // keep updated hot rows before they lose their slots
        e = launch_flush(h, s);
        if (e != hipSuccess) return hip_fail(h, e, "build_cache(flush)");
        h->dirty = false;
    }
    if (accumulate == 0) {
        e = launch_fill_u32(h, s, h->buf.counts, h->N, 0u);
        if (e != hipSuccess) return hip_fail(h, e, "build_cache(zero counts)");
    }
    if (have_stream) {
        e = launch_histogram(h, s, d_indices, d_offsets, Lp, bags_per_table);
        if (e != hipSuccess) return hip_fail(h, e, "build_cache(histogram)");
    }
    h->profiled = before + (uint64_t)Lp;
    if (accumulate == 2) return SCARS_OK;
    h->built = false;
    h->stg[0].valid = h->stg[1].valid = false;
    h->ahead.valid = false;
    e = launch_select_and_fill(h, s, k);
    if (e != hipSuccess) return hip_fail(h, e, "build_cache(select)");
    h->built = true;
    return SCARS_OK;
}

int64_t scars_cache_rows(const scars_handle* h) { return (h && h->built) ? h->k : -1; }

static int32_t check_remap_out(scars_handle* h, const scars_remap_out* o, int64_t L, const char* who) {
    if (!o || !o->n_hit_miss || (L > 0 && (!o->slot || !o->gid || !o->loc || !o->hit_pos || !o->miss_pos || !o->miss_gid)))
        return fail(h, SCARS_ERR_INVALID_ARG, std::string(who) + ": remap_out has a null array");
    if ((o->unique_miss_gid == nullptr) != (o->n_unique_miss == nullptr))
        return fail(h, SCARS_ERR_INVALID_ARG, std::string(who) + ": unique_miss_gid and n_unique_miss go together");
    return SCARS_OK;
}

// What every remap does before its kernels: argument checks, and the look-ahead / preparation bookkeeping for the
// arrays it is about to overwrite.
static int32_t remap_prologue(scars_handle* h, const int32_t* d_indices, const int32_t* d_offsets, int64_t L, int64_t B,
                              const scars_remap_out* out, hipStream_t s, const char* who) {
    int32_t rc = check_batch(h, d_indices, d_offsets, L, B, who);
    if (rc) return rc;
    if (!h->built) return fail(h, SCARS_ERR_NOT_BUILT, std::string(who) + ": build_cache has not selected a hot set");
    if ((rc = check_remap_out(h, out, L, who))) return rc;
    h->small_sorted = false;   // pieces a forward pass sorted belong to an earlier remap
    for (int a = 0; a < 2; ++a)
        if (out->loc == h->stg[a].loc) h->stg[a].valid = false;   // these arrays no longer describe a staged batch
    hipError_t e = hipSuccess;
    if (out->loc == h->ahead.loc || out->miss_gid == h->ahead.miss_gid) {
        // the fetch ahead may still be reading these arrays on the library's stream: wait for it, then drop its rows
        if ((e = pf_join(h, s)) != hipSuccess) return hip_fail(h, e, "remap(join fetch)");
        h->ahead.valid = false;
    }
    // Segments still being prepared on the side stream read the previous batch's arrays and the sort buffers.  With
    // look-ahead this call may come while the previous batch's backward pass is still to be called: then it touches
    // nothing that pass uses (no pairs, no preparation: that starts with the forward pass instead), unless it is
    // given the very arrays the preparation reads or lists each distinct missed row once (that sorts in the same buffers).
    if (!h->lookahead || out->unique_miss_gid || out->gid == h->presort_gid || out->loc == h->presort_loc) {
        e = side_join(h, s);
        if (e != hipSuccess) return hip_fail(h, e, "remap(join)");
        h->presort_valid = false;
    }
    return SCARS_OK;
}

int32_t scars_remap(scars_handle* h, const int32_t* d_indices, const int32_t* d_offsets, int64_t L, int64_t B,
                    const scars_remap_out* out, void* stream) {
    hipStream_t s = (hipStream_t)stream;
    int32_t rc = remap_prologue(h, d_indices, d_offsets, L, B, out, s, "remap");
    if (rc) return rc;
    hipError_t e = launch_remap(h, s, d_indices, d_offsets, L, B, out);
    if (e != hipSuccess) return hip_fail(h, e, "remap");
    // worth it only when a link-bound staging kernel will leave the GPU idle (misses are possible)
    if (!h->lookahead && h->presort_min_L > 0 && L >= h->presort_min_L && h->k < h->N) {
        if ((e = start_presort(h, s, d_offsets, L, B, out)) != hipSuccess) return hip_fail(h, e, "remap(backward segments)");
    }
    return SCARS_OK;
}

int32_t scars_remap_static(scars_handle* h, const int32_t* d_indices, const int32_t* d_offsets, int64_t L, int64_t B,
                           const scars_remap_out* out, void* stream) {
    hipStream_t s = (hipStream_t)stream;
    int32_t rc = remap_prologue(h, d_indices, d_offsets, L, B, out, s, "remap_static");
    if (rc) return rc;
    if (L > SCARS_REMAP_STATIC_MAX_L)
        return fail(h, SCARS_ERR_WORKSPACE, "remap_static: more than SCARS_REMAP_STATIC_MAX_L lookups; use scars_remap");
    if (out->unique_miss_gid)
        return fail(h, SCARS_ERR_INVALID_ARG, "remap_static: unique_miss_gid needs the workspace's sort buffers; use scars_remap");
    h->pairs_valid = false;   // (the pairs of an earlier scars_remap describe another batch once `out` is rewritten)
    hipError_t e = launch_remap_static(h, s, d_indices, d_offsets, L, B, out);
    if (e != hipSuccess) return hip_fail(h, e, "remap_static");
    return SCARS_OK;
}

int32_t scars_embedding_bag_fwd(scars_handle* h, const int32_t* d_indices, const int32_t* d_offsets, int64_t L,
                                int64_t B, const scars_remap_out* rm, float* d_out, void* stream) {
    int32_t rc = check_batch(h, d_indices, d_offsets, L, B, "embedding_bag_fwd");
    if (rc) return rc;
    if (!h->built) return fail(h, SCARS_ERR_NOT_BUILT, "embedding_bag_fwd: build_cache has not selected a hot set");
    if ((rc = check_remap_out(h, rm, L, "embedding_bag_fwd"))) return rc;
    if (!d_out && (int64_t)h->T * B > 0) return fail(h, SCARS_ERR_INVALID_ARG, "embedding_bag_fwd: null output");
    hipError_t e = launch_fwd(h, (hipStream_t)stream, d_offsets, L, B, rm, d_out);
    if (e != hipSuccess) return hip_fail(h, e, "embedding_bag_fwd");
    return SCARS_OK;
}

static int32_t bwd_update_impl(scars_handle* h, const int32_t* d_indices, const int32_t* d_offsets, int64_t L, int64_t B,
                               const scars_remap_out* rm, const float* d_grad_out, float lr, float eps,
                               const scars_bwd_out* out, const scars_remap_out* next_rm, const int32_t* d_next_offsets,
                               int64_t next_L, int64_t next_B, void* stream, const char* who) {
    int32_t rc = check_batch(h, d_indices, d_offsets, L, B, who);
    if (rc) return rc;
    if (!h->built) return fail(h, SCARS_ERR_NOT_BUILT, std::string(who) + ": build_cache has not selected a hot set");
    if ((rc = check_remap_out(h, rm, L, who))) return rc;
    if (!d_grad_out && L > 0) return fail(h, SCARS_ERR_INVALID_ARG, std::string(who) + ": null gradient");
    if (out && (!out->n_unique || !out->seg_start || (L > 0 && (!out->sorted_gid || !out->sorted_bag || !out->unique_gid))))
        return fail(h, SCARS_ERR_INVALID_ARG, std::string(who) + ": bwd_out has a null array");
    if (next_rm) {
        if (!h->lookahead) return fail(h, SCARS_ERR_INVALID_ARG, std::string(who) + ": SCARS_TUNE_LOOKAHEAD is off");
        if (!d_next_offsets || next_L < 0 || next_B < 0) return fail(h, SCARS_ERR_INVALID_ARG, std::string(who) + ": null or negative argument for the next batch");
        if (next_L > h->buf.max_L || (int64_t)h->T * next_B > h->buf.max_G)
            return fail(h, SCARS_ERR_WORKSPACE, std::string(who) + ": next batch larger than the bound max_L / max_G");
        if ((rc = check_remap_out(h, next_rm, next_L, who))) return rc;
        if (next_rm->unique_miss_gid) return fail(h, SCARS_ERR_INVALID_ARG, std::string(who) + ": the next batch was remapped with unique_miss_gid");
        if (next_rm->loc == rm->loc || next_rm->miss_gid == rm->miss_gid)
            return fail(h, SCARS_ERR_INVALID_ARG, std::string(who) + ": the next batch needs remap outputs of its own");
    }
    hipError_t e = side_join(h, (hipStream_t)stream);
    if (e == hipSuccess) e = launch_bwd(h, (hipStream_t)stream, d_offsets, L, B, rm, d_grad_out, lr, eps, out, next_rm, d_next_offsets, next_L, next_B);
    if (e != hipSuccess) return hip_fail(h, e, who);
    if (L > 0) h->dirty = true;
    return SCARS_OK;
}

int32_t scars_embedding_bag_bwd_update(scars_handle* h, const int32_t* d_indices, const int32_t* d_offsets,
                                       int64_t L, int64_t B, const scars_remap_out* rm, const float* d_grad_out,
                                       float lr, float eps, const scars_bwd_out* out, void* stream) {
    return bwd_update_impl(h, d_indices, d_offsets, L, B, rm, d_grad_out, lr, eps, out, nullptr, nullptr, 0, 0, stream,
                           "embedding_bag_bwd_update");
}

int32_t scars_embedding_bag_bwd_update_ahead(scars_handle* h, const int32_t* d_indices, const int32_t* d_offsets,
                                             int64_t L, int64_t B, const scars_remap_out* rm, const float* d_grad_out,
                                             float lr, float eps, const scars_bwd_out* out,
                                             const scars_remap_out* next_rm, const int32_t* d_next_offsets,
                                             int64_t next_L, int64_t next_B, void* stream) {
    if (h && !next_rm) return fail(h, SCARS_ERR_INVALID_ARG, "embedding_bag_bwd_update_ahead: null next batch");
    return bwd_update_impl(h, d_indices, d_offsets, L, B, rm, d_grad_out, lr, eps, out, next_rm, d_next_offsets, next_L,
                           next_B, stream, "embedding_bag_bwd_update_ahead");
}

int32_t scars_classify_samples(scars_handle* h, const int32_t* d_offsets, int64_t L, int64_t B, const scars_remap_out* rm,
                               const scars_classify_out* out, void* stream) {
    int32_t rc = check_batch(h, L > 0 ? (const int32_t*)d_offsets : nullptr, d_offsets, L, B, "classify_samples");
    if (rc) return rc;
    if (!h->built) return fail(h, SCARS_ERR_NOT_BUILT, "classify_samples: build_cache has not selected a hot set");
    if ((rc = check_remap_out(h, rm, L, "classify_samples"))) return rc;
    if (!out || !out->n_hot_normal || (B > 0 && (!out->is_hot || !out->hot_ids || !out->normal_ids)))
        return fail(h, SCARS_ERR_INVALID_ARG, "classify_samples: classify_out has a null array");
    hipError_t e = launch_classify(h, (hipStream_t)stream, d_offsets, L, B, rm, out);
    if (e != hipSuccess) return hip_fail(h, e, "classify_samples");
    return SCARS_OK;
}

int32_t scars_partition_batch(scars_handle* h, const int32_t* d_indices, const int32_t* d_offsets, int64_t L, int64_t B,
                              const int32_t* d_ids, const int32_t* d_n, const scars_subbatch_out* out, void* stream) {
    int32_t rc = check_batch(h, d_indices, d_offsets, L, B, "partition_batch");
    if (rc) return rc;
    if (!d_n || (B > 0 && !d_ids)) return fail(h, SCARS_ERR_INVALID_ARG, "partition_batch: null sample list");
    if (!out || !out->offsets || !out->n_lookups_bags || (L > 0 && !out->indices))
        return fail(h, SCARS_ERR_INVALID_ARG, "partition_batch: subbatch_out has a null array");
    hipError_t e = launch_partition(h, (hipStream_t)stream, d_indices, d_offsets, L, B, d_ids, d_n, out);
    if (e != hipSuccess) return hip_fail(h, e, "partition_batch");
    return SCARS_OK;
}

int32_t scars_portion_usage(scars_handle* h, const int32_t* d_offsets, int64_t L, int64_t B, const scars_remap_out* rm,
                            int64_t portion_rows, int32_t n_portions, int32_t* d_usage, void* stream) {
    int32_t rc = check_batch(h, L > 0 ? (const int32_t*)d_offsets : nullptr, d_offsets, L, B, "portion_usage");
    if (rc) return rc;
    if (!h->built) return fail(h, SCARS_ERR_NOT_BUILT, "portion_usage: build_cache has not selected a hot set");
    if ((rc = check_remap_out(h, rm, L, "portion_usage"))) return rc;
    if (portion_rows < 1 || n_portions < 1 || n_portions > 64 || !d_usage)
        return fail(h, SCARS_ERR_INVALID_ARG, "portion_usage: portion_rows >= 1, 1 <= n_portions <= 64, usage not null");
    hipError_t e = launch_portion_usage(h, (hipStream_t)stream, d_offsets, L, B, rm, portion_rows, n_portions, d_usage);
    if (e != hipSuccess) return hip_fail(h, e, "portion_usage");
    return SCARS_OK;
}

// rows per count value from the device skew table, hottest class first
static int32_t load_classes(scars_handle* h, hipStream_t s, std::vector<std::pair<uint32_t, int64_t>>* classes) {
    hipError_t e = launch_count_of_counts(h, s);
    if (e != hipSuccess) return hip_fail(h, e, "plan(count of counts)");
    std::vector<uint32_t> host(kPlanBins + kPlanBigCap + 4);
    e = hipMemcpyAsync(host.data(), h->ws.plan_cc, host.size() * 4, hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return hip_fail(h, e, "plan(copy)");
    const uint32_t n_big = host[kPlanBins + kPlanBigCap];
    if (n_big > (uint32_t)kPlanBigCap) return fail(h, SCARS_ERR_WORKSPACE, "plan: too many rows with a count of 65536 or more");
    std::vector<uint32_t> big(host.begin() + kPlanBins, host.begin() + kPlanBins + n_big);
    std::sort(big.begin(), big.end(), std::greater<uint32_t>());
    classes->clear();
    for (size_t i = 0; i < big.size();) {
        size_t j = i;
        while (j < big.size() && big[j] == big[i]) ++j;
        classes->push_back({big[i], (int64_t)(j - i)});
        i = j;
    }
    for (int c = kPlanBins - 1; c >= 0; --c)
        if (host[c]) classes->push_back({(uint32_t)c, (int64_t)host[c]});
    return SCARS_OK;
}

static int32_t check_plan(scars_handle* h, const scars_plan_in* in) {
    if (!h) return SCARS_ERR_INVALID_ARG;
    if (!h->bound) return fail(h, SCARS_ERR_WORKSPACE, "plan: no buffers bound");
    if (!in || !(in->device_params > 0.0) || !(in->per_sample_params > 0.0) || !(in->samples_per_epoch > 0.0) ||
        in->profile_samples < 1)
        return fail(h, SCARS_ERR_INVALID_ARG, "plan: parameters must be positive");
    return SCARS_OK;
}

int32_t scars_epoch_cost(scars_handle* h, const scars_plan_in* in, int64_t k, double* cost, double* batch, void* stream) {
    int32_t rc = check_plan(h, in);
    if (rc) return rc;
    if (k < 0 || k > h->N || !cost) return fail(h, SCARS_ERR_INVALID_ARG, "epoch_cost: k out of range or null output");
    std::vector<std::pair<uint32_t, int64_t>> classes;
    if ((rc = load_classes(h, (hipStream_t)stream, &classes))) return rc;
    double b = 0.0;
    const double c = plan_cost(classes, h->T, in->profile_samples, k, in->device_params, in->per_sample_params, (double)h->D,
                               in->samples_per_epoch, &b);
    if (batch) *batch = b;
    if (!std::isfinite(c)) return fail(h, SCARS_ERR_INVALID_ARG, "epoch_cost: no room for a batch of one sample (b < 1)");
    *cost = c;
    return SCARS_OK;
}

int32_t scars_caching_gain(scars_handle* h, const scars_plan_in* in, int64_t k, double* lhs, double* t1, void* stream) {
    int32_t rc = check_plan(h, in);
    if (rc) return rc;
    if (k < 0 || k >= h->N || !lhs || !t1) return fail(h, SCARS_ERR_INVALID_ARG, "caching_gain: k out of range or null output");
    const double M = in->device_params, a = in->per_sample_params, d = (double)h->D;
    const double b = (M - (double)k * d) / a, b2 = b - d / a;
    if (!(b2 >= 1.0)) return fail(h, SCARS_ERR_INVALID_ARG, "caching_gain: no room for a batch of one sample with one more row cached");
    std::vector<std::pair<uint32_t, int64_t>> classes;
    if ((rc = load_classes(h, (hipStream_t)stream, &classes))) return rc;
    // rows are ranked by count: the first k are cached, the next one is e', the rest stay outside C'
    double sum = 0.0, pe = 0.0;
    int64_t before = 0;
    for (const auto& cl : classes) {
        const int64_t cached = std::min<int64_t>(std::max<int64_t>(k + 1 - before, 0), cl.second);
        const double p = std::min(1.0, (double)cl.first / (double)in->profile_samples);
        if (before <= k && k < before + cl.second) pe = p;       // e' is in this class
        before += cl.second;
        const int64_t rest = cl.second - cached;
        if (rest > 0 && cl.first > 0)
            sum += (double)rest * (b * (1.0 - std::pow(1.0 - p, b2)) - b2 * (1.0 - std::pow(1.0 - p, b))) / b2;
    }
    *lhs = 1.0 - std::pow(1.0 - pe, b);
    *t1 = sum;
    return SCARS_OK;
}

int32_t scars_plan_cache(scars_handle* h, const scars_plan_in* in, scars_plan_out* out, void* stream) {
    int32_t rc = check_plan(h, in);
    if (rc) return rc;
    if (!out) return fail(h, SCARS_ERR_INVALID_ARG, "plan_cache: null output");
    std::vector<std::pair<uint32_t, int64_t>> classes;
    if ((rc = load_classes(h, (hipStream_t)stream, &classes))) return rc;
    const double M = in->device_params, a = in->per_sample_params, d = (double)h->D, Q = in->samples_per_epoch;
    // feasible k: b = (M - k d) / a >= 1
    const double kf = std::floor((M - a) / d);
    if (kf < 0.0) return fail(h, SCARS_ERR_INVALID_ARG, "plan_cache: the device cannot hold a batch of one sample");
    const int64_t k_max = (int64_t)std::min<double>((double)h->N, kf);
    auto cost = [&](int64_t k, double* b) { return plan_cost(classes, h->T, in->profile_samples, k, M, a, d, Q, b); };
    int64_t best_k = 0;
    double best_b = 0.0, best = cost(0, &best_b);
    auto consider = [&](int64_t k) {
        double b;
        const double c = cost(k, &b);
        if (c < best || (c == best && k < best_k)) { best = c; best_k = k; best_b = b; }
    };
    if (k_max <= 4096) {
        for (int64_t k = 1; k <= k_max; ++k) consider(k);           // small tables: every k
    } else {
        // class borders, then three rounds of a 64-point grid narrowing around the best point
        int64_t before = 0;
        for (const auto& cl : classes) {
            before += cl.second;
            if (before <= k_max && classes.size() <= 4096) consider(before);
        }
        int64_t lo = 0, hi = k_max;
        for (int round = 0; round < 4; ++round) {
            const int64_t step = std::max<int64_t>(1, (hi - lo) / 64);
            for (int64_t k = lo; k <= hi; k += step) consider(k);
            consider(hi);
            lo = std::max<int64_t>(0, best_k - step);
            hi = std::min<int64_t>(k_max, best_k + step);
        }
    }
    out->best_k = best_k;
    out->best_cost = best;
    out->best_batch = best_b;
    out->cost_no_cache = cost(0, &out->batch_no_cache);
    out->k_max = k_max;
    return SCARS_OK;
}

int32_t scars_flush_cache(scars_handle* h, void* stream) {
    if (!h) return SCARS_ERR_INVALID_ARG;
    if (!h->bound) return fail(h, SCARS_ERR_WORKSPACE, "flush_cache: no buffers bound");
    if (!h->built) return fail(h, SCARS_ERR_NOT_BUILT, "flush_cache: nothing cached");
    hipError_t e = pf_join(h, (hipStream_t)stream);
    if (e == hipSuccess) e = launch_flush(h, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(h, e, "flush_cache");
    h->dirty = false;
    return SCARS_OK;
}

int32_t scars_sync_status(scars_handle* h, void* stream) {
    if (!h) return SCARS_ERR_INVALID_ARG;
    if (!h->bound) return fail(h, SCARS_ERR_WORKSPACE, "sync_status: no buffers bound");
    hipStream_t s = (hipStream_t)stream;
    int32_t st[4] = {0, 0, 0, 0};
    hipError_t e = side_join(h, s);   // side-stream kernels latch errors too
    if (e == hipSuccess) e = pf_join(h, s);
    // scars_remap_static latches into the status word of the library's static array (shared by every handle on this GPU)
    int32_t* const st2_dev = static_status_if_used();
    int32_t st2[4] = {0, 0, 0, 0};
    if (e == hipSuccess) e = hipMemcpyAsync(st, h->ws.status, sizeof(st), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess && st2_dev) e = hipMemcpyAsync(st2, st2_dev, sizeof(st2), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return hip_fail(h, e, "sync_status");
    if (st[0] != 0 || st2[0] != 0) {
        if (st[0] != 0) e = launch_fill_u32(h, s, (uint32_t*)h->ws.status, 4, 0u);
        if (e == hipSuccess && st2[0] != 0) e = launch_fill_u32(h, s, (uint32_t*)st2_dev, 4, 0u);
        if (e == hipSuccess) e = hipStreamSynchronize(s);
        if (e != hipSuccess) return hip_fail(h, e, "sync_status(clear)");
        const int32_t code = st[0] != 0 ? st[0] : st2[0];
        return fail(h, code, code == SCARS_ERR_INDEX_RANGE ? "device: index out of range" : "device: bad offsets");
    }
    return SCARS_OK;
}

const char* scars_last_error(const scars_handle* h) { return h ? h->err.c_str() : "null handle"; }

int32_t scars_host_alloc(int64_t bytes, void** out) {
    if (!out || bytes <= 0) return SCARS_ERR_INVALID_ARG;
    *out = nullptr;
    hipError_t e = hipHostMalloc(out, (size_t)bytes, hipHostMallocDefault);
    if (e != hipSuccess) {
        (void)hipGetLastError();   // a refused allocation must not be reported again by the next launch's error check
        *out = nullptr;
        return SCARS_ERR_HIP;
    }
    return SCARS_OK;
}

int32_t scars_host_free(void* p) {
    if (!p) return SCARS_ERR_INVALID_ARG;
    return hipHostFree(p) == hipSuccess ? SCARS_OK : SCARS_ERR_HIP;
}

int32_t scars_memcpy(void* dst, const void* src, int64_t bytes, int32_t kind, void* stream) {
    if (!dst || !src || bytes < 0 || kind < 1 || kind > 3) return SCARS_ERR_INVALID_ARG;
    const hipMemcpyKind k = kind == 1 ? hipMemcpyHostToDevice : (kind == 2 ? hipMemcpyDeviceToHost : hipMemcpyDeviceToDevice);
    return hipMemcpyAsync(dst, src, (size_t)bytes, k, (hipStream_t)stream) == hipSuccess ? SCARS_OK : SCARS_ERR_HIP;
}

int32_t scars_calibration_copy(void* d_dst, const void* d_src, int64_t bytes, void* stream) {
    if (!d_dst || !d_src || bytes < 0 || bytes % 16 != 0) return SCARS_ERR_INVALID_ARG;
    return launch_calib_copy((hipStream_t)stream, d_dst, d_src, bytes) == hipSuccess ? SCARS_OK : SCARS_ERR_HIP;
}

int32_t scars_calibration_read(const void* d_src, int64_t bytes, void* d_sink, void* stream) {
    if (!d_src || !d_sink || bytes < 0 || bytes % 16 != 0) return SCARS_ERR_INVALID_ARG;
    return launch_calib_read((hipStream_t)stream, d_src, bytes, d_sink) == hipSuccess ? SCARS_OK : SCARS_ERR_HIP;
}

int32_t scars_calibration_link(void* h_pinned, int64_t host_bytes, void* d_buf, int64_t n_granules, int32_t granule_bytes,
                               int32_t scattered, int32_t to_host, int32_t workgroups, void* stream) {
    if (!h_pinned || !d_buf || n_granules < 0 || workgroups < 1 || workgroups > 65536) return SCARS_ERR_INVALID_ARG;
    if (granule_bytes != 16 && granule_bytes != 32 && granule_bytes != 64 && granule_bytes != 128 && granule_bytes != 256 &&
        granule_bytes != 512 && granule_bytes != 1024)
        return SCARS_ERR_INVALID_ARG;
    if (host_bytes < granule_bytes) return SCARS_ERR_INVALID_ARG;
    if (n_granules == 0) return SCARS_OK;
    return launch_calib_link((hipStream_t)stream, h_pinned, host_bytes, d_buf, n_granules, granule_bytes, scattered != 0,
                             to_host != 0, workgroups) == hipSuccess ? SCARS_OK : SCARS_ERR_HIP;
}

int32_t scars_profile_enable(scars_handle* h, int32_t on) {
    if (!h) return SCARS_ERR_INVALID_ARG;
    h->profile = on != 0;
    return SCARS_OK;
}

int32_t scars_profile_read(scars_handle* h, void* stream, scars_kernel_time* out, int32_t cap, int32_t* n_out) {
    if (!h || !n_out || cap < 0 || (cap > 0 && !out)) return SCARS_ERR_INVALID_ARG;
    hipError_t e = hipStreamSynchronize((hipStream_t)stream);
    if (e == hipSuccess && h->side) e = hipStreamSynchronize(h->side);
    if (e == hipSuccess && h->pool_stream) e = hipStreamSynchronize(h->pool_stream);
    if (e != hipSuccess) return hip_fail(h, e, "profile_read");
    std::vector<scars_kernel_time> acc;
    // an update and the fetch enqueued beside it on the library's stream carry the same tag: did they run together?
    struct Pair { hipEvent_t ua = nullptr, ub = nullptr, fa = nullptr, fb = nullptr; };
    std::map<int64_t, Pair> pairs;
    for (auto& p : h->timer.pending) {
        if (p.tag <= 0) continue;
        if (std::strcmp(p.name, "fetch_ahead") == 0) { pairs[p.tag].fa = p.a; pairs[p.tag].fb = p.b; }
        else if (std::strncmp(p.name, "seg_rows", 8) == 0) { pairs[p.tag].ua = p.a; pairs[p.tag].ub = p.b; }
    }
    for (auto& kv : pairs) {
        const Pair& q = kv.second;
        if (!q.ua || !q.fa) continue;
        float u = 0.f, f = 0.f, d = 0.f;     // update and fetch durations, fetch start relative to update start (ms)
        if (hipEventElapsedTime(&u, q.ua, q.ub) != hipSuccess || hipEventElapsedTime(&f, q.fa, q.fb) != hipSuccess ||
            hipEventElapsedTime(&d, q.ua, q.fa) != hipSuccess)
            continue;
        const float overlap = std::min(d + f, u) - std::max(d, 0.f);
        ++h->n_ahead_timed;
        if (overlap < 0.25f * std::min(u, f)) ++h->n_ahead_serial;
    }
    for (auto& p : h->timer.pending) {
        float ms = 0.f;
        (void)hipEventElapsedTime(&ms, p.a, p.b);
        (void)hipEventDestroy(p.a);
        (void)hipEventDestroy(p.b);
        bool found = false;
        for (auto& r : acc)
            if (std::strcmp(r.name, p.name) == 0) { r.launches += 1; r.total_ms += ms; found = true; break; }
        if (!found) acc.push_back({p.name, 1, (double)ms});
    }
    h->timer.pending.clear();
    const int32_t n = (int32_t)std::min<size_t>(acc.size(), (size_t)cap);
    for (int32_t i = 0; i < n; ++i) out[i] = acc[i];
    *n_out = n;
    return SCARS_OK;
}

}  // extern "C"
