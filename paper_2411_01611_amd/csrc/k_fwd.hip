// embedding_bag_fwd: fetch of missed rows over the host link, then the pooled gather-sum.
//
// Fig. 1 of the paper: per-sample embeddings are looked up in main memory and sent to the GPU; Section II-B:
// rows of the cached set C are already on the device.  Here the misses of a batch are first copied, row by
// row, from the pinned host tables into a staging area in HBM (the only kernel that touches the host
// link), after which every lookup -- hit or miss -- is a 16-byte-per-lane gather from HBM.  A row of R bytes
// is read by R/16 lanes ("group"); a wave holds 64/(R/16) groups.  Short bags: one group per bag.  Long
// bags: one wave per bag, its groups striding over the bag and combining by a fixed shuffle tree.  The
// order of additions depends only on positions, never on where a row came from.
#include "scars_dev.h"

namespace scars {

constexpr int kStageBlocks = 128;  // workgroups of the staging kernel
constexpr int kAheadBlocks = 128;  // ... when it fetches ahead, beside the update kernel (64 and 512 are slower)
constexpr int kPoolUnroll = 8;   // rows in flight per lane group when pooling
constexpr int kShortTailUnroll = 2;   // the same for lookups after the first of a short bag: few registers, more waves

// ---- staging of missed rows ---------------------------------------------------------------------------
// (stage_rows_body in scars_dev.h; the backward pass can carry the same job in its update launch)
// flag 1 = the row may be fetched ahead (k_mark_ahead), so want = 1 fetches ahead and want = 0 fetches what was left out.
__global__ __launch_bounds__(kBlock) void k_stage_misses(const Meta* __restrict__ meta, StageArgs S) {
    __shared__ int32_t s_rbase[SCARS_MAX_TABLES + 1];
    stage_rows_body((int)blockIdx.x, (int)gridDim.x, meta, s_rbase, S);
}

// The same launch with, in its first T workgroups, the per-table sort of the batch's (row, bag) pairs that its backward
// pass will need (small batches of a caller who has stated the lookups per table): the sort reads what remap wrote and
// nothing of the fetch, and takes about as long as the fetch of a small batch's missed rows takes on the host link.
__global__ __launch_bounds__(kBlock) void k_stage_misses_sort(const Meta* __restrict__ meta, StageArgs S, int T, SmallSortArgs Q) {
    if ((int)blockIdx.x < T) {
        small_sort_body((int)blockIdx.x, meta, Q);
    } else {
        __shared__ int32_t s_rbase[SCARS_MAX_TABLES + 1];
        stage_rows_body((int)blockIdx.x - T, (int)gridDim.x - T, meta, s_rbase, S);
    }
}

// Fetching the NEXT batch's missed rows while the current batch's backward pass runs: a row may be fetched now unless
// that pass writes it.  Its distinct rows `excl[0..n_excl)` are sorted, so a binary search tells; this kernel only
// sets the flags (it touches no host memory, so it is not slowed by the link), k_stage_misses then fetches the
// flagged rows, and the next batch's forward pass the others once the update is done.  A row is never read while
// it may be written.
__global__ __launch_bounds__(kBlock) void k_mark_ahead(const int32_t* __restrict__ miss_gid, const int32_t* __restrict__ d_count,
                                                       const int32_t* __restrict__ excl, const int32_t* __restrict__ d_n_excl,
                                                       uint8_t* __restrict__ flags, int64_t cap_rows) {
    const int64_t n = min((int64_t)*d_count, cap_rows);
    const int32_t ne = max(min(*d_n_excl, (int32_t)cap_rows), 0);
    for (int64_t j = (int64_t)blockIdx.x * kBlock + threadIdx.x; j < n; j += (int64_t)gridDim.x * kBlock) {
        const int32_t gid = miss_gid[j];
        int32_t lo = 0, hi = ne;                 // first position with excl[pos] >= gid
        while (lo < hi) {
            const int32_t mid = (lo + hi) >> 1;
            if (excl[mid] < gid) lo = mid + 1; else hi = mid;
        }
        flags[j] = (lo < ne && excl[lo] == gid) ? 0 : 1;
    }
}

// ---- pooled sum -------------------------------------------------------------------------------------
template <int DTYPE> struct Chunk;   // one 16-byte piece of a row, as fp32 accumulators

template <> struct Chunk<SCARS_DTYPE_F32> {
    static constexpr int kVals = 4;
    float v[4];
    __device__ __forceinline__ void zero() { v[0] = v[1] = v[2] = v[3] = 0.f; }
    __device__ __forceinline__ void add(const uint4& r) {
        v[0] += __uint_as_float(r.x); v[1] += __uint_as_float(r.y);
        v[2] += __uint_as_float(r.z); v[3] += __uint_as_float(r.w);
    }
};

template <> struct Chunk<SCARS_DTYPE_BF16> {
    static constexpr int kVals = 8;
    float v[8];
    __device__ __forceinline__ void zero() {
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = 0.f;
    }
    __device__ __forceinline__ void add(const uint4& r) {
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] += __uint_as_float(w[i] << 16);             // low half = even element
            v[2 * i + 1] += __uint_as_float(w[i] & 0xFFFF0000u);
        }
    }
};

typedef float f32x4 __attribute__((ext_vector_type(4)));

// The pooled sums are written once and not read again by this launch: streaming stores keep them out of the way of
// the rows the caches hold (one index per bag, 872 MB of sums per launch: 0.68 -> 0.78 of peak; long bags: 0.81 -> 0.84).
template <int DTYPE>
__device__ __forceinline__ void store_chunk(const Chunk<DTYPE>& acc, float* __restrict__ out, int64_t g, int D, int c) {
    f32x4* o = (f32x4*)(out + g * D + (int64_t)c * Chunk<DTYPE>::kVals);
#pragma unroll
    for (int q = 0; q < Chunk<DTYPE>::kVals / 4; ++q) {
        const f32x4 v = {acc.v[4 * q], acc.v[4 * q + 1], acc.v[4 * q + 2], acc.v[4 * q + 3]};
        __builtin_nontemporal_store(v, o + q);
    }
}

// Sum of the rows at positions [a, b) by one group of LPR lanes (lane c holds 16-byte piece c of the row).
// The group's lanes fetch LPR locations with one load and hand them out by shuffles, so the row addresses of a
// whole window are known before the first row arrives; positions are added in order.
template <int DTYPE, int LPR, int UNROLL>
__device__ __forceinline__ void pool_range(Chunk<DTYPE>& acc, int32_t a, int32_t b, const int32_t* __restrict__ loc,
                                           const uint4* __restrict__ cache, const uint4* __restrict__ staging, int32_t k,
                                           int chunks, int c, bool lane_on) {
    const int gl0 = (lane_id() / LPR) * LPR;                     // first lane of this group inside the wave
    for (int32_t w0 = a; w0 < b; w0 += LPR) {
        const int32_t n = min((int32_t)LPR, b - w0);
        const int32_t lv = c < n ? loc[w0 + c] : -1;
        for (int base = 0; base < n; base += UNROLL) {
            uint4 row[UNROLL];
            bool on[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const int i = base + u;
                const int32_t l = __shfl(lv, gl0 + (i & (LPR - 1)), kWave);
                on[u] = lane_on && i < n && l >= 0;
                if (on[u]) {
                    const uint4* p = l < k ? cache + (int64_t)l * chunks : staging + (int64_t)(l - k) * chunks;
                    row[u] = p[c];
                }
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u)
                if (on[u]) acc.add(row[u]);
        }
    }
}

// one group of LPR lanes per bag
template <int DTYPE, int LPR>
__global__ __launch_bounds__(kBlock) void k_pool_group(const int32_t* __restrict__ off, int64_t G, int32_t L,
                                                       const int32_t* __restrict__ loc, const uint4* __restrict__ cache,
                                                       const uint4* __restrict__ staging, int32_t k, int chunks, int D,
                                                       float* __restrict__ out) {
    const int64_t g = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / LPR;
    const int c = threadIdx.x % LPR;
    if (g >= G) return;
    const int32_t a = min(max(off[g], 0), L);
    const int32_t b = min(max(off[g + 1], a), L);
    Chunk<DTYPE> acc;
    acc.zero();
    pool_range<DTYPE, LPR, kPoolUnroll>(acc, a, b, loc, cache, staging, k, chunks, c, c < chunks);
    if (c < chunks) store_chunk<DTYPE>(acc, out, g, D, c);
}

// Bags of one or two lookups (one index per sample and table): a group has nothing to overlap inside a bag, so
// it takes kShortBags bags at once -- their offsets, then their first locations, then their first rows are
// each fetched together.  Lookups beyond the first of a bag are added afterwards, in order.  Swept 2 / 4 / 8 bags:
// 4 for large batches (1.7 M bags: 0.75 / 0.78 / 0.68 of peak), 2 for small ones (53 k bags: 0.51 / 0.43 / 0.31).
constexpr int64_t kShortFewBags = 1 << 18;   // below this many bags: 2 at once, so that there are more workgroups

template <int DTYPE, int LPR, int kShortBags>
__global__ __launch_bounds__(kBlock) void k_pool_short(const int32_t* __restrict__ off, int64_t G, int32_t L,
                                                       const int32_t* __restrict__ loc, const uint4* __restrict__ cache,
                                                       const uint4* __restrict__ staging, int32_t k, int chunks, int D,
                                                       float* __restrict__ out, int filter) {
    // filter 0: every bag.  1: only bags that need no staged row (empty, or one lookup that hit the cache): these do
    // not depend on the fetch of the missed rows.  2: only the other bags.
    const int64_t TG = (G + kShortBags - 1) / kShortBags;        // groups; group gi takes bags gi, gi + TG, ...
    const int64_t gi = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / LPR;
    const int c = threadIdx.x % LPR;
    if (gi >= TG) return;
    const bool lane_on = c < chunks;
    int32_t a[kShortBags], b[kShortBags], l0[kShortBags];
#pragma unroll
    for (int q = 0; q < kShortBags; ++q) {
        const int64_t g = gi + q * TG;
        a[q] = b[q] = 0;
        if (g < G) {
            a[q] = min(max(off[g], 0), L);
            b[q] = min(max(off[g + 1], a[q]), L);
        }
    }
#pragma unroll
    for (int q = 0; q < kShortBags; ++q) l0[q] = b[q] > a[q] ? loc[a[q]] : -1;
    bool take[kShortBags];
#pragma unroll
    for (int q = 0; q < kShortBags; ++q) {
        const bool no_staged = b[q] - a[q] <= 1 && l0[q] < k;     // (an invalid lookup has location -1)
        take[q] = gi + q * TG < G && (filter == 0 || (filter == 1) == no_staged);
    }
    uint4 row[kShortBags];
#pragma unroll
    for (int q = 0; q < kShortBags; ++q) {
        if (take[q] && lane_on && l0[q] >= 0) {
            const uint4* p = l0[q] < k ? cache + (int64_t)l0[q] * chunks : staging + (int64_t)(l0[q] - k) * chunks;
            row[q] = p[c];
        }
    }
#pragma unroll
    for (int q = 0; q < kShortBags; ++q) {
        const int64_t g = gi + q * TG;
        if (!take[q]) continue;
        Chunk<DTYPE> acc;
        acc.zero();
        if (lane_on && l0[q] >= 0) acc.add(row[q]);
        if (b[q] - a[q] > 1) pool_range<DTYPE, LPR, kShortTailUnroll>(acc, a[q] + 1, b[q], loc, cache, staging, k, chunks, c, lane_on);
        if (lane_on) store_chunk<DTYPE>(acc, out, g, D, c);
    }
}

// The bags k_pool_short leaves out under filter 1 (they need a staged row, or hold several lookups), for batches in
// which such bags are few: one lane per bag reads its offsets and first location, the wave ballots the bags to do
// and its 64/LPR lane groups take them 64/LPR at a time.  A launch with a lane group per bag would spend its time
// on the bags it skips.  Same sums as k_pool_short: positions added in order, starting from zero.
template <int DTYPE, int LPR>
__global__ __launch_bounds__(kBlock) void k_pool_short_rest(const int32_t* __restrict__ off, int64_t G, int32_t L,
                                                            const int32_t* __restrict__ loc, const uint4* __restrict__ cache,
                                                            const uint4* __restrict__ staging, int32_t k, int chunks, int D,
                                                            float* __restrict__ out) {
    constexpr int NG = kWave / LPR;
    const int64_t g = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    int32_t a = 0, b = 0;
    if (g < G) {
        a = min(max(off[g], 0), L);
        b = min(max(off[g + 1], a), L);
    }
    const int32_t l0 = b > a ? loc[a] : -1;
    const bool take = g < G && !(b - a <= 1 && l0 < k);          // the complement of filter 1
    uint64_t m = ballot64(take);                                  // the same in every lane
    const int q = lane_id() / LPR, c = lane_id() % LPR;
    const bool lane_on = c < chunks;
    const int64_t g0 = g - lane_id();                             // the wave's first bag
    while (m) {
        int src = -1;                                             // the lane that owns this group's bag of the round
#pragma unroll
        for (int j = 0; j < NG; ++j) {
            if (m) {
                const int l = __ffsll((long long)m) - 1;
                m &= m - 1;
                if (q == j) src = l;
            }
        }
        const int sl = max(src, 0);
        const int32_t aa = __shfl(a, sl, kWave), bb = __shfl(b, sl, kWave);
        if (src >= 0) {
            Chunk<DTYPE> acc;
            acc.zero();
            pool_range<DTYPE, LPR, kShortTailUnroll>(acc, aa, bb, loc, cache, staging, k, chunks, c, lane_on);
            if (lane_on) store_chunk<DTYPE>(acc, out, g0 + src, D, c);
        }
    }
}

// one wave per bag; its 64/LPR groups take every (64/LPR)-th lookup and combine by a shuffle tree
template <int DTYPE, int LPR>
__global__ __launch_bounds__(kBlock) void k_pool_wave(const int32_t* __restrict__ off, int64_t G, int32_t L,
                                                      const int32_t* __restrict__ loc, const uint4* __restrict__ cache,
                                                      const uint4* __restrict__ staging, int32_t k, int chunks, int D,
                                                      float* __restrict__ out) {
    constexpr int NG = kWave / LPR;
    const int64_t g = (int64_t)blockIdx.x * (kBlock / kWave) + wave_id();
    if (g >= G) return;
    const int q = lane_id() / LPR, c = lane_id() % LPR;
    const int32_t a = min(max(off[g], 0), L);
    const int32_t b = min(max(off[g + 1], a), L);
    Chunk<DTYPE> acc;
    acc.zero();
    const bool lane_on = c < chunks;
    // the bag's locations are fetched 64 at a time with one coalesced load and handed out by shuffles, so
    // every row address is known before the first row arrives
    for (int32_t w0 = a; w0 < b; w0 += kWave) {
        const int32_t n = min(kWave, b - w0);
        const int32_t lv = lane_id() < n ? loc[w0 + lane_id()] : -1;
        for (int base = 0; base < n; base += NG * kPoolUnroll) {   // same trip count for every lane
            uint4 row[kPoolUnroll];
            bool on[kPoolUnroll];
#pragma unroll
            for (int u = 0; u < kPoolUnroll; ++u) {
                const int i = base + q + u * NG;
                const int32_t l = __shfl(lv, i & (kWave - 1), kWave);
                on[u] = lane_on && i < n && l >= 0;
                if (on[u]) {
                    const uint4* p = l < k ? cache + (int64_t)l * chunks : staging + (int64_t)(l - k) * chunks;
                    row[u] = p[c];
                }
            }
#pragma unroll
            for (int u = 0; u < kPoolUnroll; ++u)
                if (on[u]) acc.add(row[u]);
        }
    }
#pragma unroll
    for (int d = kWave / 2; d >= LPR; d >>= 1) {
#pragma unroll
        for (int i = 0; i < Chunk<DTYPE>::kVals; ++i) acc.v[i] += __shfl_down(acc.v[i], d, 64);
    }
    if (q == 0 && c < chunks) store_chunk<DTYPE>(acc, out, g, D, c);
}

template <int DTYPE, int LPR>
static void launch_pool_t(hipStream_t s, int mode, const int32_t* off, int64_t G, int64_t L, const int32_t* loc,
                          const void* cache, const void* staging, int64_t k, int chunks, int D, float* out, int filter) {
    if (mode == 2 && filter == 2) {
        hipLaunchKernelGGL((k_pool_short_rest<DTYPE, LPR>), dim3((unsigned)div_up(G, kBlock)), dim3(kBlock), 0, s, off, G,
                           (int32_t)L, loc, (const uint4*)cache, (const uint4*)staging, (int32_t)k, chunks, D, out);
    } else if (mode == 2) {
        const int bags = G < kShortFewBags ? 2 : 4;
        const int64_t TG = div_up(G, bags);
        if (bags == 2)
            hipLaunchKernelGGL((k_pool_short<DTYPE, LPR, 2>), dim3((unsigned)div_up(TG * LPR, kBlock)), dim3(kBlock), 0, s, off,
                               G, (int32_t)L, loc, (const uint4*)cache, (const uint4*)staging, (int32_t)k, chunks, D, out, filter);
        else
            hipLaunchKernelGGL((k_pool_short<DTYPE, LPR, 4>), dim3((unsigned)div_up(TG * LPR, kBlock)), dim3(kBlock), 0, s, off,
                               G, (int32_t)L, loc, (const uint4*)cache, (const uint4*)staging, (int32_t)k, chunks, D, out, filter);
    } else if (mode == 1) {
        hipLaunchKernelGGL((k_pool_wave<DTYPE, LPR>), dim3((unsigned)div_up(G, kBlock / kWave)), dim3(kBlock), 0, s, off,
                           G, (int32_t)L, loc, (const uint4*)cache, (const uint4*)staging, (int32_t)k, chunks, D, out);
    } else {
        hipLaunchKernelGGL((k_pool_group<DTYPE, LPR>), dim3((unsigned)div_up(G * LPR, kBlock)), dim3(kBlock), 0, s, off,
                           G, (int32_t)L, loc, (const uint4*)cache, (const uint4*)staging, (int32_t)k, chunks, D, out);
    }
}

template <int DTYPE>
static void launch_pool_d(int lpr, hipStream_t s, int mode, const int32_t* off, int64_t G, int64_t L,
                          const int32_t* loc, const void* cache, const void* staging, int64_t k, int chunks, int D,
                          float* out, int filter) {
    switch (lpr) {
#define SCARS_CASE(N) case N: launch_pool_t<DTYPE, N>(s, mode, off, G, L, loc, cache, staging, k, chunks, D, out, filter); break;
        SCARS_CASE(1) SCARS_CASE(2) SCARS_CASE(4) SCARS_CASE(8) SCARS_CASE(16) SCARS_CASE(32) SCARS_CASE(64)
#undef SCARS_CASE
    }
}

// The library's second stream (default priority, created when buffers are first bound): pooling beside the fetch in the forward pass,
// and the fetch for the next batch beside the update in the backward pass; the two uses never overlap in time.
hipError_t ensure_pool_stream(scars_handle* h) {
    hipError_t e = hipSuccess;   // (a call that failed half way is completed by the next one)
    if (!h->pool_stream) e = hipStreamCreateWithFlags(&h->pool_stream, hipStreamNonBlocking);
    for (hipEvent_t* ev : {&h->ev_pool_fork, &h->ev_pool_join, &h->ev_pf_fork, &h->ev_pf_done})
        if (e == hipSuccess && !*ev) e = hipEventCreateWithFlags(ev, hipEventDisableTiming);
    return e;
}

hipError_t launch_fwd(scars_handle* h, hipStream_t s, const int32_t* off, int64_t L, int64_t B,
                      const scars_remap_out* rm, float* out) {
    const int chunks = h->R / 16;
    const int lpr = std::min(64, next_pow2_host(chunks));
    const int64_t G = (int64_t)h->T * B;
    // rows of this batch that were fetched ahead sit in their own staging area, the others are fetched now
    hipError_t e0 = pf_join(h, s);
    if (e0 != hipSuccess) return e0;
    const bool ahead = h->ahead.valid && h->ahead.loc == rm->loc && !rm->unique_miss_gid && L > 0 && h->k < h->N;
    const int area = ahead ? h->ahead.area : 0;
    if (ahead) ++h->n_ahead_used;
    h->ahead.valid = false;
    void* const staging = h->ws.staging[area];
    for (int a = 0; a < 2; ++a)
        if (a == area || h->stg[a].loc == rm->loc) h->stg[a].valid = false;
    h->stg[area].valid = L > 0 && h->k < h->N;
    h->stg[area].loc = rm->loc;
    // 2: bags of one or two lookups, several bags per lane group; 1: long bags, a wave per bag; 0: a group per bag
    const int mode = L < 2 * G ? 2 : ((lpr < 64 && L >= G * 2 * (kWave / lpr)) ? 1 : 0);
    auto pool = [&](hipStream_t st, int filter, const char* name) {
        Timed t(h, st, name);
        if (h->dtype == SCARS_DTYPE_F32)
            launch_pool_d<SCARS_DTYPE_F32>(lpr, st, mode, off, G, L, rm->loc, h->buf.cache, staging, h->k, chunks,
                                           h->D, out, filter);
        else
            launch_pool_d<SCARS_DTYPE_BF16>(lpr, st, mode, off, G, L, rm->loc, h->buf.cache, staging, h->k, chunks,
                                            h->D, out, filter);
    };
    // With the side-stream option and short bags, the bags that need no staged row (the hits of a one-index-per-bag
    // batch) are pooled on the side stream while the missed rows are still being fetched; the rest follow the fetch.
    const bool split = mode == 2 && G > 0 && h->presort_min_L > 0 && L >= h->presort_min_L && h->k < h->N;
    if (split) {   // a stream of its own: the side stream may still be busy with the backward pass's sort
        hipError_t e = ensure_pool_stream(h);
        if (e != hipSuccess) return e;
        if ((e = hipEventRecord(h->ev_pool_fork, s)) != hipSuccess) return e;
        if ((e = hipStreamWaitEvent(h->pool_stream, h->ev_pool_fork, 0)) != hipSuccess) return e;
        pool(h->pool_stream, 1, "pool_short");
        if ((e = hipEventRecord(h->ev_pool_join, h->pool_stream)) != hipSuccess) return e;
    }
    // remap left this batch's (row, bag) pairs for the backward pass, and the caller has stated how many lookups a
    // table gets at most: each table's piece is sorted in the first workgroups of the fetch's launch
    const bool sort_here = L > 0 && h->k < h->N && h->small_sort_applies() && h->pairs_valid && h->pairs_gid == rm->gid &&
                           h->pairs_off == off && h->pairs_L == L && h->pairs_B == B;
    h->small_sorted = false;
    if (L > 0 && h->k < h->N) {   // with every row cached there can be no miss
        Timed t(h, s, sort_here ? "stage_misses+small_sort" : "stage_misses");
        const int gpb = kBlock / lpr;
        // 128 workgroups hold far more than the host link needs in flight (128 x 256 lanes x 4 x 16 bytes = 2 MB) and
        // leave half the compute units, and most wave slots, to work on other streams while this kernel waits on the
        // link (kernels sharing a compute unit with it run several times slower: its host reads fill the memory queues)
        const int grid = (int)std::max<int64_t>(1, std::min<int64_t>(div_up(L, (int64_t)gpb * kStageUnroll), ahead ? 16 * kStageBlocks : kStageBlocks));
        // (after a fetch ahead only a few rows are left: many workgroups walk the flags quickly)
        // one row per missed lookup, or (after a coalescing remap) one per distinct missed row
        const int32_t* list = rm->unique_miss_gid ? rm->unique_miss_gid : rm->miss_gid;
        const int32_t* count = rm->unique_miss_gid ? rm->n_unique_miss : rm->n_hit_miss + 1;
        const StageArgs S{list, count, (u32x4*)staging, chunks, lpr, h->buf.max_L,
                          ahead ? h->ws.fetched : (const uint8_t*)nullptr, 0};
        if (sort_here) {
            SmallSortArgs Q = small_sort_args(h, h->ws.key_buf, h->ws.val_buf, off, L, B);
            // ... and leave the runs for an update by position (cold rows from the staging area this launch fills);
            // in the look-ahead order the update needs the list of the batch's distinct rows instead
            h->small_runs = !h->lookahead;
            h->small_runs_staged = true;
            if (h->small_runs) Q.run = small_run_args(h, rm, true);
            hipLaunchKernelGGL(k_stage_misses_sort, dim3(grid + h->T), dim3(kBlock), 0, s, h->ws.meta, S, h->T, Q);
            h->small_sorted = true;
            h->small_gid = rm->gid; h->small_off = off; h->small_L = L; h->small_B = B;
        } else {
            hipLaunchKernelGGL(k_stage_misses, dim3(grid), dim3(kBlock), 0, s, h->ws.meta, S);
        }
    }
    if (G > 0) pool(s, split ? 2 : 0, split ? "pool_short_staged" : (mode == 2 ? "pool_short" : (mode == 1 ? "pool_wave" : "pool_group")));
    if (split) {   // the output is complete, in the caller's stream order, when this call returns
        hipError_t e = hipStreamWaitEvent(s, h->ev_pool_join, 0);
        if (e != hipSuccess) return e;
    }
    return hipGetLastError();
}

// `fused` set: nothing is launched for the fetch itself; *fused receives the job (and *fused_blocks its workgroups)
// for the caller to carry in its own launch on stream s.  Otherwise the fetch runs on the library's second stream.
hipError_t launch_fetch_ahead(scars_handle* h, hipStream_t s, const scars_remap_out* next_rm, int64_t next_L,
                              const int32_t* excl, const int32_t* n_excl, int area, StageArgs* fused, int* fused_blocks) {
    hipError_t e = hipSuccess;
    const int chunks = h->R / 16;
    const int lpr = std::min(64, next_pow2_host(chunks));
    const int gpb = kBlock / lpr;
    // (rows of 128 bytes need twice the workgroups to keep as many bytes in flight: 4.30 -> 4.10 ms per step on the
    // bf16 workload, together with more workgroups for the update beside it)
    // (rows of 512 bytes: 192 beside 768 workgroups of the update against 128 beside 512: 4.57 -> 4.54 ms per step with
    // most of the batch's rows cold, 1.25 -> 1.23 with one row in five cold)
    const int ahead_blocks = h->R <= 128 ? 2 * kAheadBlocks : (h->R >= 512 ? kAheadBlocks * 3 / 2 : kAheadBlocks);
    const int grid = (int)std::max<int64_t>(1, std::min<int64_t>(div_up(next_L, (int64_t)gpb * kStageUnroll), ahead_blocks));
    {   // on the caller's stream, before the update kernel: beside that kernel it would crawl (see k_stage_misses)
        Timed t(h, s, "mark_ahead");
        const int mgrid = (int)std::max<int64_t>(1, std::min<int64_t>(div_up(next_L, kBlock), 256 * 8));
        hipLaunchKernelGGL(k_mark_ahead, dim3(mgrid), dim3(kBlock), 0, s, next_rm->miss_gid, next_rm->n_hit_miss + 1,
                           excl, n_excl, h->ws.fetched, h->buf.max_L);
    }
    const StageArgs S{next_rm->miss_gid, next_rm->n_hit_miss + 1, (u32x4*)h->ws.staging[area], chunks, lpr, h->buf.max_L,
                      h->ws.fetched, 1};
    if (fused) {
        *fused = S;
        *fused_blocks = grid;
    } else {
        if ((e = ensure_pool_stream(h)) != hipSuccess) return e;
        hipStream_t const pf = h->pool_stream;
        if ((e = hipEventRecord(h->ev_pf_fork, s)) != hipSuccess) return e;
        if ((e = hipStreamWaitEvent(pf, h->ev_pf_fork, 0)) != hipSuccess) return e;
        {
            Timed t(h, pf, "fetch_ahead");
            hipLaunchKernelGGL(k_stage_misses, dim3(grid), dim3(kBlock), 0, pf, h->ws.meta, S);
        }
        if ((e = hipGetLastError()) != hipSuccess) return e;
        if ((e = hipEventRecord(h->ev_pf_done, pf)) != hipSuccess) return e;
        h->pf_pending = true;
    }
    h->stg[area].valid = false;
    h->ahead.valid = true;
    h->ahead.loc = next_rm->loc;
    h->ahead.miss_gid = next_rm->miss_gid;
    h->ahead.area = area;
    return hipGetLastError();
}

}  // namespace scars
