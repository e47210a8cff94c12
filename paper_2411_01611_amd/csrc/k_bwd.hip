// embedding_bag_bwd_update: sorted-segment scatter-add of the upstream gradient and the row update.
//
// Section IV of the paper splits an iteration into forward, backward and optimization and attributes the
// cost of the last two to writes of embedding rows (device memory for cached rows, host DRAM for the
// rest).  Here: (1) pairs (gid, bag) in position order; (2) stable radix sort by gid; (3) segment heads by
// ordered compaction (the integer outputs); (4) one lane group per distinct row sums its run of
// gradient rows and applies the update, with the row fetched while the gradients stream in; (5) a run of
// more than 64 lookups is summed per 64-position chunk into fp64 partials, which a following launch adds in
// chunk order.  No floating-point atomics: results are bit-stable.
#include "scars_dev.h"

namespace scars {

// ---- (1) pairs ----------------------------------------------------------------------------------------
// (bag_pairs in scars_dev.h; scars_remap may already have written them in the launch that lists hits and misses)
__global__ __launch_bounds__(kBlock) void k_bwd_pairs(const int32_t* __restrict__ gid, const int32_t* __restrict__ off,
                                                      int32_t L, int64_t G, int lpb, int shift,
                                                      uint32_t* __restrict__ key, uint32_t* __restrict__ val) {
    bag_pairs((int64_t)blockIdx.x, gid, off, L, G, lpb, shift, key, val);
}

__global__ void k_bwd_empty(int32_t* __restrict__ n_unique, int32_t* __restrict__ seg_start) {
    if (threadIdx.x == 0) { n_unique[0] = 0; n_unique[1] = 0; seg_start[0] = 0; }
}

// ---- (3) segment heads ----------------------------------------------------------------------------------
constexpr int kPerWaveS = kScanTile / (kBlock / kWave);
constexpr int kRoundsS = kPerWaveS / kWave;

__device__ __forceinline__ bool is_head(const uint32_t* __restrict__ key, int64_t j, int64_t L) {
    if (j >= L) return false;
    const uint32_t k = key[j];
    if (k == 0xFFFFFFFFu) return false;
    return j == 0 || key[j - 1] != k;
}

// per tile: number of heads and number of valid (non-sentinel) keys
__global__ __launch_bounds__(kBlock) void k_seg_count(const uint32_t* __restrict__ key, int64_t L,
                                                      uint32_t* __restrict__ blk_head, uint32_t* __restrict__ blk_valid) {
    __shared__ uint32_t s_a[4], s_b[4];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + wave_id() * kPerWaveS;
    uint32_t nh = 0, nv = 0;
#pragma unroll
    for (int r = 0; r < kRoundsS; ++r) {
        const int64_t j = base + r * kWave + lane_id();
        nh += (uint32_t)__popcll(ballot64(is_head(key, j, L)));
        nv += (uint32_t)__popcll(ballot64(j < L && key[j] != 0xFFFFFFFFu));
    }
    if (lane_id() == 0) { s_a[wave_id()] = nh; s_b[wave_id()] = nv; }
    __syncthreads();
    if (threadIdx.x == 0) {
        blk_head[blockIdx.x] = s_a[0] + s_a[1] + s_a[2] + s_a[3];
        blk_valid[blockIdx.x] = s_b[0] + s_b[1] + s_b[2] + s_b[3];
    }
}

__global__ __launch_bounds__(kBlock) void k_seg_scan(uint32_t* __restrict__ a, uint32_t* __restrict__ b, int n,
                                                     int32_t* __restrict__ n_unique) {
    __shared__ uint32_t s_scan[8];
    uint32_t ca, cb;
    scan_two_counts(a, b, n, s_scan, &ca, &cb);
    if (threadIdx.x == 0) { n_unique[0] = (int32_t)ca; n_unique[1] = (int32_t)cb; }
}

// Run starts by ordered compaction; per run also where the update kernel finds the row and its first gradient row.
// A pair's value holds the bag and the lookup's place inside it (bag_pairs), so the first lookup of a run is at
// position off[bag] + place, and loc[] there is what remap found for it: the cache slot, or the copy of a cold row its
// forward pass staged.  Two dependent loads from arrays the size of the batch, no search and no probe of the dense
// row map.  (When the place saturated, or the offsets were bad, the map is probed and a cold row read from host memory.)
__global__ __launch_bounds__(kBlock) void k_seg_write(const uint32_t* __restrict__ key, const uint32_t* __restrict__ val,
                                                      int64_t L, const uint32_t* __restrict__ blk_head,
                                                      const uint32_t* __restrict__ blk_valid, int scanned,
                                                      int32_t* __restrict__ n_unique, int32_t* __restrict__ seg_start,
                                                      int32_t* __restrict__ unique_gid, int32_t* __restrict__ sorted_gid,
                                                      int32_t* __restrict__ sorted_bag, int32_t* __restrict__ chunk_run,
                                                      const int32_t* __restrict__ slot_of, uint32_t N,
                                                      int32_t* __restrict__ unique_slot, uint32_t* __restrict__ first_bag,
                                                      const int32_t* __restrict__ off, int64_t G, const int32_t* __restrict__ gid_of,
                                                      const int32_t* __restrict__ loc_of, int32_t k, int staged, int shift, int via_loc) {
    __shared__ uint32_t s_a[4], s_red[8];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + wave_id() * kPerWaveS;
    const uint32_t sat = (1u << shift) - 1u;
    bool hd[kRoundsS];
    uint32_t kk[kRoundsS], vv[kRoundsS];
    uint32_t nh = 0;
    // stage 1: keys (and their left neighbours) and values of all rounds
#pragma unroll
    for (int r = 0; r < kRoundsS; ++r) {
        const int64_t j = base + r * kWave + lane_id();
        hd[r] = is_head(key, j, L);
        kk[r] = j < L ? key[j] : 0xFFFFFFFFu;
        vv[r] = j < L ? val[j] : 0u;
        nh += (uint32_t)__popcll(ballot64(hd[r]));
    }
    if (lane_id() == 0) s_a[wave_id()] = nh;
    // stage 2: per run start, the start of its first bag and/or the row's slot in the dense map.  via_loc: the slot is
    // not probed (a random access into an array of N entries) unless the place inside the bag is unknown (it saturated);
    // stage 3 takes it from what remap found for the run's first lookup.  That pays while the batch's own arrays stay in
    // the caches (655 k lookups, rows partly cold: 27 -> 20 us); for a batch of 4.3 M lookups it is three scattered
    // reads instead of one (50 -> 92 us), so there only the cold rows go through stage 3.
    int32_t src[kRoundsS], p0[kRoundsS];
#pragma unroll
    for (int r = 0; r < kRoundsS; ++r) {
        const bool h = hd[r] && kk[r] < N;
        const uint32_t bag = vv[r] >> shift;
        const bool placed = h && (int64_t)bag < G && (vv[r] & sat) < sat && (via_loc || staged);
        p0[r] = placed ? off[bag] : -1;
        src[r] = (h && !(placed && via_loc)) ? slot_of[kk[r]] : -1;
    }
    // stage 3: the run's first lookup: its location (cache slot, or the staged copy of a cold row).  The pairs were
    // built from these very offsets, so the position is the lookup's own; should the offsets not describe the batch
    // (a latched error, outputs unspecified) the location read is still one remap wrote for this batch, hence a valid
    // cache slot or staging row.  In the cold-rows-only form the row id at that position is checked as well.
#pragma unroll
    for (int r = 0; r < kRoundsS; ++r) {
        if (hd[r] && p0[r] >= 0 && (via_loc || src[r] < 0)) {
            const int64_t p = (int64_t)p0[r] + (vv[r] & sat);
            if (p < L) {
                const int32_t l = loc_of[p];
                if (via_loc) {
                    src[r] = (l < k || staged) ? l : -1;      // without a staged copy a cold row is read from host memory
                } else if ((uint32_t)gid_of[p] == kk[r] && l >= k) {
                    src[r] = l;
                }
            } else if (via_loc) {
                src[r] = slot_of[kk[r]];
            }
        }
    }
    __syncthreads();
    uint32_t before, bv, n_runs, n_valid;
    const bool last = tile_prefix2(blk_head, blk_valid, blockIdx.x, gridDim.x, scanned != 0, s_red, n_unique, &before, &bv,
                                   &n_runs, &n_valid);
    // one entry past the last run start: the number of valid pairs
    if (last && threadIdx.x == 0) seg_start[n_runs] = (int32_t)n_valid;
    if (scanned && blockIdx.x == 0 && threadIdx.x == 0) seg_start[n_unique[0]] = n_unique[1];
    for (int w = 0; w < wave_id(); ++w) before += s_a[w];
#pragma unroll
    for (int r = 0; r < kRoundsS; ++r) {
        const int64_t j = base + r * kWave + lane_id();
        const uint64_t m = ballot64(hd[r]);
        if (hd[r]) {
            const uint32_t u = before + (uint32_t)rank_below(m);
            seg_start[u] = (int32_t)j;
            unique_gid[u] = (int32_t)kk[r];
            // for the update kernel: where the row lives and which gradient row comes first, so that it can
            // issue the row fetch and the first gradient fetch at once
            unique_slot[u] = src[r];
            first_bag[u] = vv[r] >> shift;
        }
        // each round is one chunk of kLongRunMin (= 64) positions: remember which run its first position is in
        if (lane_id() == 0 && j < L) chunk_run[j / kLongRunMin] = (int32_t)(before + (hd[r] ? 1u : 0u)) - 1;
        before += (uint32_t)__popcll(m);
        if (sorted_gid && j < L) {   // caller asked for the sorted pairs as well
            sorted_gid[j] = (int32_t)kk[r];
            sorted_bag[j] = (int32_t)(vv[r] >> shift);
        }
    }
}

// The same outputs for a batch whose tables were each sorted by a workgroup of their own (k_small_sort): table t's
// sorted piece lies at the piece's own place in kin / vin, and the tables' numbers of valid pairs and of distinct rows
// are known, so one workgroup per table can place its piece in the final order (valid pairs of all tables first, in
// table order; invalid ones behind them) and list its run starts at once: no counting launch, no tile prefix.
__global__ __launch_bounds__(kBlock) void k_small_segments(const uint32_t* __restrict__ kin, const uint32_t* __restrict__ vin,
                                                           const int32_t* __restrict__ off, int64_t B, int32_t L, int T, int limit,
                                                           const uint32_t* __restrict__ tab_valid,
                                                           const uint32_t* __restrict__ tab_heads,
                                                           uint32_t* __restrict__ kout, uint32_t* __restrict__ vout,
                                                           int32_t* __restrict__ n_unique, int32_t* __restrict__ seg_start,
                                                           int32_t* __restrict__ unique_gid, int32_t* __restrict__ sorted_gid,
                                                           int32_t* __restrict__ sorted_bag, int32_t* __restrict__ chunk_run,
                                                           const int32_t* __restrict__ slot_of, uint32_t N,
                                                           int32_t* __restrict__ unique_slot, uint32_t* __restrict__ first_bag,
                                                           int64_t G, const int32_t* __restrict__ gid_of,
                                                           const int32_t* __restrict__ loc_of, int32_t k, int staged, int shift,
                                                           int via_loc) {
    constexpr int R = kSmallSortCap / kBlock;
    constexpr int kW = kBlock / kWave;
    __shared__ uint32_t s_red[kW][5];
    __shared__ uint32_t s_a[kW];
    const int t = blockIdx.x, w = wave_id(), lane = lane_id();
    // over the tables: valid pairs and distinct rows before this table and in all, invalid pairs before this table
    uint32_t acc[5] = {0u, 0u, 0u, 0u, 0u};
    for (int i = threadIdx.x; i < T; i += kBlock) {
        int32_t ai, ni;
        bool oi;
        small_piece(off, B, L, i, limit, &ai, &ni, &oi);
        const uint32_t vi = min(tab_valid[i], (uint32_t)ni), hi = min(tab_heads[i], vi);
        acc[1] += vi;
        acc[4] += hi;
        if (i < t) { acc[0] += vi; acc[2] += (uint32_t)ni - vi; acc[3] += hi; }
    }
#pragma unroll
    for (int j = 0; j < 5; ++j) {
        acc[j] = wave_sum(acc[j]);
        if (lane == 0) s_red[w][j] = acc[j];
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 5; ++j) {
        acc[j] = 0;
#pragma unroll
        for (int ww = 0; ww < kW; ++ww) acc[j] += s_red[ww][j];
    }
    const uint32_t base = acc[0], valid_all = acc[1], tail = acc[1] + acc[2], heads_before = acc[3], heads_all = acc[4];
    int32_t a, n;
    bool over;
    small_piece(off, B, L, t, limit, &a, &n, &over);
    const uint32_t nv = min(tab_valid[t], (uint32_t)n);
    const uint32_t sat = (1u << shift) - 1u;
    const int rounds = (n + kBlock - 1) / kBlock;           // the piece dealt out as in k_small_sort
    const int per_wave = rounds * kWave;
    bool hd[R];
    uint32_t kk[R], vv[R];
    uint32_t nh = 0;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int q = w * per_wave + r * kWave + lane;
        const bool in = r < rounds && q < n;
        kk[r] = in ? kin[a + q] : 0xFFFFFFFFu;
        vv[r] = in ? vin[a + q] : 0u;
        hd[r] = in && (uint32_t)q < nv && kk[r] != 0xFFFFFFFFu && (q == 0 || kin[a + q - 1] != kk[r]);
        nh += (uint32_t)__popcll(ballot64(hd[r]));
    }
    if (lane == 0) s_a[w] = nh;
    // where the update finds each run's row: the two stages of k_seg_write
    int32_t src[R], p0[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const bool h = hd[r] && kk[r] < N;
        const uint32_t bag = vv[r] >> shift;
        const bool placed = h && (int64_t)bag < G && (vv[r] & sat) < sat && (via_loc || staged);
        p0[r] = placed ? off[bag] : -1;
        src[r] = (h && !(placed && via_loc)) ? slot_of[kk[r]] : -1;
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        if (hd[r] && p0[r] >= 0 && (via_loc || src[r] < 0)) {
            const int64_t p = (int64_t)p0[r] + (vv[r] & sat);
            if (p < L) {
                const int32_t l = loc_of[p];
                if (via_loc) {
                    src[r] = (l < k || staged) ? l : -1;
                } else if ((uint32_t)gid_of[p] == kk[r] && l >= k) {
                    src[r] = l;
                }
            } else if (via_loc) {
                src[r] = slot_of[kk[r]];
            }
        }
    }
    __syncthreads();
    uint32_t before = heads_before;
    for (int ww = 0; ww < w; ++ww) before += s_a[ww];
    const uint64_t le = lane == 63 ? ~0ull : ((1ull << (lane + 1)) - 1ull);
#pragma unroll
    for (int r = 0; r < R; ++r) {
        if (r >= rounds) continue;                            // (the same for every lane of the workgroup)
        const int q = w * per_wave + r * kWave + lane;
        const bool in = q < n;
        const uint64_t m = ballot64(hd[r]);
        const uint32_t j = (uint32_t)q < nv ? base + (uint32_t)q : tail + ((uint32_t)q - nv);   // final position
        if (in) {
            kout[j] = kk[r];
            vout[j] = vv[r];
            if (sorted_gid) {
                sorted_gid[j] = (int32_t)kk[r];
                sorted_bag[j] = (int32_t)(vv[r] >> shift);
            }
            // a chunk of kLongRunMin positions remembers which run its first position is in
            if (j % kLongRunMin == 0)
                chunk_run[j / kLongRunMin] = (uint32_t)q < nv ? (int32_t)(before + (uint32_t)__popcll(m & le)) - 1
                                                              : (int32_t)heads_all - 1;
        }
        if (hd[r]) {
            const uint32_t u = before + (uint32_t)rank_below(m);
            seg_start[u] = (int32_t)j;
            unique_gid[u] = (int32_t)kk[r];
            unique_slot[u] = src[r];
            first_bag[u] = vv[r] >> shift;
        }
        before += (uint32_t)__popcll(m);
    }
    if (t == T - 1 && threadIdx.x == 0) {
        seg_start[heads_all] = (int32_t)valid_all;
        n_unique[0] = (int32_t)heads_all;
        n_unique[1] = (int32_t)valid_all;
    }
}

// ---- (4)/(5) segment reduce and update --------------------------------------------------------------------
struct UpdateArgs {
    const Meta* meta;
    const int32_t* slot_of;
    void* cache;
    float* state_cache;
    float lr, eps;
    int D;
    const void* staging;  // rows fetched by the forward pass of this batch (null when not usable)
    int32_t k;       // cached rows: a source index >= k is row (index - k) of the staging area
    uint32_t N;      // rows in all tables: a key at or above it is never dereferenced
    uint32_t Gm1;    // last bag: bag ids are clamped to it (both only matter after an offsets error)
    int shift;       // a pair's value is (bag << shift) | place inside the bag
};

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Where a row lives: cache slot (HBM) or pinned host table; the Adagrad accumulator beside it.
template <int DTYPE, int OPT>
struct RowRef {
    void* w;          // where the updated row is written
    const void* wr;   // where its current value is read
    float* s;
    // src: cache slot in [0, k); k + i = cold row whose current value is row i of the staging area (the copy the
    // forward pass of this batch fetched, so the host link carries only the write); -1 = cold row read from host
    __device__ __forceinline__ void locate(const UpdateArgs& A, const int32_t* s_rbase, int T, int32_t gid, int32_t src) {
        s = nullptr;
        constexpr int kElem = DTYPE == SCARS_DTYPE_F32 ? 4 : 2;
        if (src >= 0 && src < A.k) {
            w = (char*)A.cache + (int64_t)src * A.D * kElem;
            wr = w;
            if (OPT == SCARS_OPT_ADAGRAD) s = A.state_cache + (int64_t)src * A.D;
        } else {
            const int t = upper_table(s_rbase, T, gid);
            const int64_t row = gid - s_rbase[t];
            w = (char*)A.meta->table[t] + row * A.D * kElem;
            wr = (src >= A.k && A.staging) ? (const void*)((const char*)A.staging + (int64_t)(src - A.k) * A.D * kElem) : w;
            if (OPT == SCARS_OPT_ADAGRAD) s = A.meta->state[t] + row * A.D;
        }
    }
    // lane owns columns [4c, 4c+4).  A row and its accumulator are read once per launch, the gradient rows beside them
    // about once per lookup of their bag: streaming loads keep the former from pushing the latter out of the caches
    // (every row cached, 20 lookups a bag: step 0.387 -> 0.360 ms; one index per bag: unchanged).
    __device__ __forceinline__ void load(int c, float (&wv)[4], float (&sv)[4]) const {
        if (DTYPE == SCARS_DTYPE_F32) {
            const f32x4 v = __builtin_nontemporal_load((const f32x4*)wr + c);
            wv[0] = v.x; wv[1] = v.y; wv[2] = v.z; wv[3] = v.w;
        } else {
            const u32x2 v = __builtin_nontemporal_load((const u32x2*)wr + c);
            wv[0] = __uint_as_float(v.x << 16); wv[1] = __uint_as_float(v.x & 0xFFFF0000u);
            wv[2] = __uint_as_float(v.y << 16); wv[3] = __uint_as_float(v.y & 0xFFFF0000u);
        }
        if (OPT == SCARS_OPT_ADAGRAD) {
            const f32x4 v = __builtin_nontemporal_load((const f32x4*)s + c);
            sv[0] = v.x; sv[1] = v.y; sv[2] = v.z; sv[3] = v.w;
        }
    }
    // One optimizer step with summed gradient g, evaluated in fp64 and rounded once.  From a zero accumulator
    // Adagrad's step is lr*g/(|g|+eps), whose slope in g reaches lr/eps, so an fp32-accurate g would miss a
    // 1e-6 absolute bar; hence fp64 sums and fp64 arithmetic here.
    __device__ __forceinline__ void step_and_store(const UpdateArgs& A, int c, const float (&wv)[4], const float (&sv)[4],
                                                   const double (&g)[4]) const {
        const double lr = (double)A.lr, eps = (double)A.eps;
        double wn[4];
        if (OPT == SCARS_OPT_SGD) {
#pragma unroll
            for (int i = 0; i < 4; ++i) wn[i] = (double)wv[i] - lr * g[i];
        } else {
            double st[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                st[i] = (double)sv[i] + g[i] * g[i];
                wn[i] = (double)wv[i] - lr * g[i] / (sqrt(st[i]) + eps);
            }
            const f32x4 o = {(float)st[0], (float)st[1], (float)st[2], (float)st[3]};
            __builtin_nontemporal_store(o, (f32x4*)s + c);
        }
        // A row is written once per launch and not read again by it: streaming stores (measured against ordinary
        // ones: steps with cold rows 1-2 % shorter, the 53 k-lookup batch 6 %, nothing slower).
        if (DTYPE == SCARS_DTYPE_F32) {
            const f32x4 o = {(float)wn[0], (float)wn[1], (float)wn[2], (float)wn[3]};
            __builtin_nontemporal_store(o, (f32x4*)w + c);
        } else {
            const u32x2 o = {(uint32_t)f32_to_bf16((float)wn[0]) | ((uint32_t)f32_to_bf16((float)wn[1]) << 16),
                             (uint32_t)f32_to_bf16((float)wn[2]) | ((uint32_t)f32_to_bf16((float)wn[3]) << 16)};
            __builtin_nontemporal_store(o, (u32x2*)w + c);
        }
    }
};

constexpr int kLongRun = kLongRunMin;   // runs up to this many lookups are summed by one lane group
constexpr int kGradUnroll = 4;  // gradient rows in flight per lane group in the per-row kernel
constexpr int kTaskUnroll = 16;  // ... and in a task of a long run (few groups, long chains: go wide)
constexpr int kCombUnroll = 16; // partial sums in flight when a long run is combined
constexpr int64_t kFusedWideMaxL = 1 << 17;   // shared launch: batches up to this size take the wide long-run part

// Sum of the gradient rows val[j], j in [p0, p1), columns [4c, 4c+4), in position order, fp64.  The group's lanes
// fetch a window of bag ids with one load and hand them out by shuffles, so every gradient row address of a trip is
// known at once (bag ids and rows are otherwise two dependent round trips per trip); UNROLL rows in flight.  Every
// lane of the group must call, also lanes beyond the row (c >= dq: they read the last piece and their sums are
// never stored).  Indices are clamped instead of guarded so that the loads are issued back to back.
template <int LPG, int UNROLL>
__device__ __forceinline__ void sum_grads(const uint32_t* __restrict__ val, const float4* __restrict__ g4, int dq, int c,
                                          int32_t p0, int32_t p1, uint32_t Gm1, int shift, double (&acc)[4]) {
    constexpr int W = LPG < kWave ? LPG : kWave;                 // positions one load of the group covers
    const int wl = LPG < kWave ? c : lane_id();                  // this lane's place in the window
    const int gl0 = LPG < kWave ? (lane_id() / LPG) * LPG : 0;   // first lane of the group inside the wave
    const int cc = min(c, dq - 1);
    for (int32_t w0 = p0; w0 < p1; w0 += W) {
        const int32_t n = min((int32_t)W, p1 - w0);
        const uint32_t bv = min(val[min(w0 + wl, p1 - 1)] >> shift, Gm1);
        for (int base = 0; base < n; base += UNROLL) {
            float4 gv[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const uint32_t bag = __shfl(bv, gl0 + min(base + u, n - 1), kWave);
                gv[u] = g4[(int64_t)bag * dq + cc];
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                if (base + u < n) {
                    acc[0] += (double)gv[u].x; acc[1] += (double)gv[u].y; acc[2] += (double)gv[u].z; acc[3] += (double)gv[u].w;
                }
            }
        }
    }
}

// One lane group per distinct row whose run has at most kLongRun lookups; the row (and accumulator) is
// fetched while the gradient rows stream in.  Longer runs are left to k_seg_long.
// `block` of `nblocks` workgroups share the rows (the kernel's own grid, or the part of a fused grid that does this).
template <int DTYPE, int OPT, int LPG>
__device__ __forceinline__ void seg_rows_body(int block, int nblocks, const uint32_t* __restrict__ val,
                                              const int32_t* __restrict__ n_unique, const int32_t* __restrict__ seg_start,
                                              const int32_t* __restrict__ unique_gid, const int32_t* __restrict__ unique_slot,
                                              const uint32_t* __restrict__ first_bag, const float* __restrict__ grad,
                                              const UpdateArgs& A) {
    __shared__ int32_t s_rbase[SCARS_MAX_TABLES + 1];
    const int T = A.meta->num_tables;
    for (int t = threadIdx.x; t <= T; t += kBlock) s_rbase[t] = A.meta->row_base[t];
    __syncthreads();
    const int32_t U = n_unique[0];
    const int c = threadIdx.x % LPG;
    const int dq = A.D / 4;
    const bool lane_on = c < dq;              // lanes beyond the row stay: they hand out bag ids in sum_grads
    const int cc = min(c, dq - 1);
    const float4* g4 = (const float4*)grad;
    const int64_t ngroups = (int64_t)nblocks * (kBlock / LPG);
    for (int64_t r = (int64_t)block * (kBlock / LPG) + threadIdx.x / LPG; r < U; r += ngroups) {
        const int32_t a = seg_start[r], b = seg_start[r + 1];
        const uint32_t gid = (uint32_t)unique_gid[r];
        const int32_t slot = unique_slot[r];
        const uint32_t bag0 = min(first_bag[r], A.Gm1);
        if (b - a > kLongRun || gid >= A.N) continue;
        // the row, its accumulator and the first gradient row are all addressable now: one round trip
        RowRef<DTYPE, OPT> ref;
        ref.locate(A, s_rbase, T, (int32_t)gid, slot);
        float wv[4], sv[4] = {0.f, 0.f, 0.f, 0.f};
        ref.load(cc, wv, sv);
        const float4 g0 = g4[(int64_t)bag0 * dq + cc];
        double acc[4] = {(double)g0.x, (double)g0.y, (double)g0.z, (double)g0.w};
        if (b - a > 1) sum_grads<LPG, kGradUnroll>(val, g4, dq, c, a + 1, b, A.Gm1, A.shift, acc);
        if (lane_on) ref.step_and_store(A, c, wv, sv, acc);
    }
}

template <int DTYPE, int OPT, int LPG>
__global__ __launch_bounds__(kBlock) void k_seg_rows(const uint32_t* __restrict__ val, const int32_t* __restrict__ n_unique,
                                                     const int32_t* __restrict__ seg_start, const int32_t* __restrict__ unique_gid,
                                                     const int32_t* __restrict__ unique_slot, const uint32_t* __restrict__ first_bag,
                                                     const float* __restrict__ grad, UpdateArgs A) {
    seg_rows_body<DTYPE, OPT, LPG>((int)blockIdx.x, (int)gridDim.x, val, n_unique, seg_start, unique_gid, unique_slot, first_bag,
                                   grad, A);
}

// Runs longer than kLongRun, first half: one lane group per chunk of kLongRun sorted positions.  Such a run
// overlaps a chunk either by covering its first position ("side 0") or by starting inside it and running past
// its end ("side 1"); at most one of each per chunk.  The overlap is summed into partial[chunk][side].
// chunk_run[ch] is the run that holds the chunk's first position.  Independent of k_seg_rows.
template <int LPG, int UNROLL>
__device__ __forceinline__ void seg_long_body(int block, int nblocks, const uint32_t* __restrict__ key,
                                              const uint32_t* __restrict__ val, const int32_t* __restrict__ n_unique,
                                              const int32_t* __restrict__ seg_start, const int32_t* __restrict__ chunk_run,
                                              const float* __restrict__ grad, double* __restrict__ partial, int D, uint32_t Gm1, int shift) {
    const int32_t Lv = n_unique[1];
    const int c = threadIdx.x % LPG;
    const bool lane_on = c * 4 < D;
    const int dq = D / 4;
    const float4* g4 = (const float4*)grad;
    constexpr int gpb = kBlock / LPG;
    const int64_t ngroups = (int64_t)nblocks * gpb;
    const int32_t nchunks = (Lv + kLongRun - 1) / kLongRun;
    for (int64_t ch = (int64_t)block * gpb + threadIdx.x / LPG; ch < nchunks; ch += ngroups) {
        const int32_t j0 = (int32_t)ch * kLongRun, j1 = min(j0 + kLongRun, Lv);
        const uint32_t k0 = key[j0], k1 = key[j1 - 1];
        const uint32_t kp = j0 > 0 ? key[j0 - 1] : ~k0;
        const uint32_t kn = j1 < Lv ? key[j1] : ~k1;
        const int32_t r0 = chunk_run[ch];
        const int32_t r1 = j1 < Lv ? chunk_run[ch + 1] : 0;
        for (int side = 0; side < 2; ++side) {
            // a long run over this chunk must continue across one of its borders
            const bool cand = side == 0 ? (kp == k0 || kn == k0) : (k1 != k0 && kn == k1);
            if (!cand) continue;              // (the same for every lane of the group)
            const int32_t r = side == 0 ? r0 : r1;
            const int32_t a = seg_start[r], b = seg_start[r + 1];
            if (b - a <= kLongRun) continue;
            double acc[4] = {0.0, 0.0, 0.0, 0.0};
            sum_grads<LPG, UNROLL>(val, g4, dq, c, max(a, j0), min(b, j1), Gm1, shift, acc);
            if (lane_on) {
                double* p = partial + ((int64_t)ch * 2 + side) * D + c * 4;
                p[0] = acc[0]; p[1] = acc[1]; p[2] = acc[2]; p[3] = acc[3];
            }
        }
    }
}

template <int LPG>
__global__ __launch_bounds__(kBlock) void k_seg_long(const uint32_t* __restrict__ key, const uint32_t* __restrict__ val,
                                                     const int32_t* __restrict__ n_unique, const int32_t* __restrict__ seg_start,
                                                     const int32_t* __restrict__ chunk_run, const float* __restrict__ grad,
                                                     double* __restrict__ partial, int D, uint32_t Gm1, int shift) {
    seg_long_body<LPG, kTaskUnroll>((int)blockIdx.x, (int)gridDim.x, key, val, n_unique, seg_start, chunk_run, grad, partial, D, Gm1, shift);
}

// Runs longer than kLongRun when none can be very long (the caller has stated how many lookups a table gets at most,
// and a run lies inside one table): the workgroup of the chunk in which such a run starts sums the whole run, a piece
// per lane group, adds the pieces in LDS in group order and applies the update.  No partial sums in memory and no
// second launch, which is what counts for the small batches that statement is made for.  Any run length is summed
// correctly; a long one only takes longer (its positions divided by the workgroup's lane groups, in sequence).
// One workgroup per chunk; every branch below is taken by the whole workgroup.
// The run [a, b) of row gid (found at `slot`, as RowRef::locate reads it), by the whole workgroup.
template <int DTYPE, int OPT, int LPG, int UNROLL>
__device__ __forceinline__ void whole_run_apply(int32_t a, int32_t b, uint32_t gid, int32_t slot, const uint32_t* __restrict__ val,
                                                const float* __restrict__ grad, const UpdateArgs& A) {
    constexpr int gpb = kBlock / LPG;
    __shared__ double s_sum[kBlock * 4];
    const int c = threadIdx.x % LPG, g = threadIdx.x / LPG;
    const int dq = A.D / 4;
    const int cc = min(c, dq - 1);
    RowRef<DTYPE, OPT> ref;
    float wv[4] = {0.f, 0.f, 0.f, 0.f}, sv[4] = {0.f, 0.f, 0.f, 0.f};
    if (g == 0) {   // the row and its accumulator come in while the gradient rows are summed
        ref.locate(A, A.meta->row_base, A.meta->num_tables, (int32_t)gid, slot);
        ref.load(cc, wv, sv);
    }
    const int32_t piece = (b - a + gpb - 1) / gpb;
    const int32_t p0 = min(a + g * piece, b), p1 = min(p0 + piece, b);
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    sum_grads<LPG, UNROLL>(val, (const float4*)grad, dq, c, p0, p1, A.Gm1, A.shift, acc);
#pragma unroll
    for (int i = 0; i < 4; ++i) s_sum[(g * LPG + c) * 4 + i] = acc[i];
    __syncthreads();
    if (g == 0 && c < dq) {
        double t[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll 2   // (unrolled in full, the loads of all groups' pieces are hoisted: up to 256 registers, for every part of the launch)
        for (int q = 0; q < gpb; ++q) {
#pragma unroll
            for (int i = 0; i < 4; ++i) t[i] += s_sum[(q * LPG + c) * 4 + i];
        }
        ref.step_and_store(A, c, wv, sv, t);
    }
}

template <int DTYPE, int OPT, int LPG, int UNROLL>
__device__ __forceinline__ void seg_whole_body(int ch, const uint32_t* __restrict__ val, const int32_t* __restrict__ n_unique,
                                               const int32_t* __restrict__ seg_start, const int32_t* __restrict__ unique_gid,
                                               const int32_t* __restrict__ unique_slot, const int32_t* __restrict__ chunk_run,
                                               const float* __restrict__ grad, const UpdateArgs& A) {
    const int32_t Lv = n_unique[1];
    const int32_t nchunks = (Lv + kLongRun - 1) / kLongRun;
    if (ch >= nchunks) return;
    const int32_t j0 = ch * kLongRun, j1 = min(j0 + kLongRun, Lv);
    // a long run that starts exactly at the chunk's first position covers the chunk; otherwise one may start inside
    // and run past the chunk's end: it then holds the next chunk's first position
    const int32_t U = n_unique[0];
    int32_t r = chunk_run[ch];
    if (r < 0 || r >= U) return;             // (only after an offsets error: nothing is dereferenced through it)
    int32_t a = seg_start[r], b = seg_start[r + 1];
    if (a != j0 || b - a <= kLongRun) {
        if (j1 >= Lv) return;
        r = chunk_run[ch + 1];
        if (r < 0 || r >= U) return;
        a = seg_start[r];
        b = seg_start[r + 1];
        if (a <= j0 || a >= j1 || b - a <= kLongRun) return;
    }
    if (b > Lv) return;
    const uint32_t gid = (uint32_t)unique_gid[r];
    if (gid >= A.N) return;
    whole_run_apply<DTYPE, OPT, LPG, UNROLL>(a, b, gid, unique_slot[r], val, grad, A);
}

// ---- the update of a small batch by position ------------------------------------------------------------------------
// After the per-table sort (small_sort_body with its run outputs) the update needs no list of runs: a lane group per
// sorted position takes the run that starts there (run_len > 0), and the workgroup of a chunk of kLongRun positions
// takes the long run that starts in the chunk, if any (at most one can: it is longer than the chunk).  Everything read
// through run_len / run_src / key is range-checked first: positions that no table's piece covers (after an offsets
// error) hold whatever an earlier batch left.  cap_staged: rows of the staging area.
__device__ __forceinline__ bool run_ok(int64_t j, int32_t len, int32_t src, uint32_t gid, int32_t L, const UpdateArgs& A,
                                       int64_t cap_staged) {
    return len > 0 && j + len <= L && gid < A.N && (src == -1 || (src >= 0 && (int64_t)src < (int64_t)A.k + cap_staged));
}

template <int DTYPE, int OPT, int LPG>
__global__ __launch_bounds__(kBlock) void k_small_update(int long_blocks, int32_t L, int64_t cap_staged,
                                                         const uint32_t* __restrict__ key, const uint32_t* __restrict__ val,
                                                         const int32_t* __restrict__ run_len, const int32_t* __restrict__ run_src,
                                                         const float* __restrict__ grad, UpdateArgs A) {
    if ((int)blockIdx.x < long_blocks) {      // one workgroup per chunk
        __shared__ int32_t s_run[4];          // position, length, source and row of the long run that starts in the chunk
        if (threadIdx.x == 0) s_run[0] = -1;
        __syncthreads();
        const int64_t p = (int64_t)blockIdx.x * kLongRun + threadIdx.x;
        if (threadIdx.x < kLongRun && p < L) {
            const int32_t len = run_len[p], src = run_src[p];
            const uint32_t gid = key[p];
            if (len > kLongRun) {             // (only after an offsets error can more than one lane get here)
                s_run[1] = len; s_run[2] = src; s_run[3] = (int32_t)gid;
                s_run[0] = (int32_t)p;
            }
        }
        __syncthreads();
        const int32_t j = s_run[0], len = s_run[1], src = s_run[2];
        const uint32_t gid = (uint32_t)s_run[3];
        if (j < 0 || len <= kLongRun || !run_ok(j, len, src, gid, L, A, cap_staged)) return;
        whole_run_apply<DTYPE, OPT, LPG, 8>(j, j + len, gid, src, val, grad, A);
        return;
    }
    __shared__ int32_t s_rbase[SCARS_MAX_TABLES + 1];
    const int T = A.meta->num_tables;
    const int64_t ngroups = (int64_t)((int)gridDim.x - long_blocks) * (kBlock / LPG);
    int64_t j = (int64_t)((int)blockIdx.x - long_blocks) * (kBlock / LPG) + threadIdx.x / LPG;
    // a lane group's first position is read while the table starts are on their way to LDS (most groups have only one)
    int32_t len = 0, src = -1;
    uint32_t gid = 0, v = 0;
    if (j < L) { len = run_len[j]; src = run_src[j]; gid = key[j]; v = val[j]; }
    for (int t = threadIdx.x; t <= T; t += kBlock) s_rbase[t] = A.meta->row_base[t];
    __syncthreads();
    const int c = threadIdx.x % LPG;
    const int dq = A.D / 4;
    const bool lane_on = c < dq;
    const int cc = min(c, dq - 1);
    const float4* g4 = (const float4*)grad;
    for (bool first = true; j < L; j += ngroups, first = false) {
        if (!first) { len = run_len[j]; src = run_src[j]; gid = key[j]; v = val[j]; }
        const uint32_t bag0 = min(v >> A.shift, A.Gm1);
        if (len > kLongRun || !run_ok(j, len, src, gid, L, A, cap_staged)) continue;
        RowRef<DTYPE, OPT> ref;
        ref.locate(A, s_rbase, T, (int32_t)gid, src);
        float wv[4], sv[4] = {0.f, 0.f, 0.f, 0.f};
        ref.load(cc, wv, sv);
        const float4 g0 = g4[(int64_t)bag0 * dq + cc];
        double acc[4] = {(double)g0.x, (double)g0.y, (double)g0.z, (double)g0.w};
        if (len > 1) sum_grads<LPG, kGradUnroll>(val, g4, dq, c, (int32_t)j + 1, (int32_t)j + len, A.Gm1, A.shift, acc);
        if (lane_on) ref.step_and_store(A, c, wv, sv, acc);
    }
}

// Both of the above in one launch: the first `long_blocks` workgroups take the chunks of long runs, the others the
// rows.  The two parts touch disjoint rows and share nothing; together the shorter one's chain of dependent memory
// round trips is hidden behind the other (a whole launch's worth of time for small batches).
// ULONG: gradient rows in flight in the long-run part.  More of them shorten its chains but cost registers, hence
// occupancy, for the whole launch: wide for small batches (a few waves per compute unit anyway), narrow for large.
// With fetch_blocks > 0 the launch carries a third, independent job in its first workgroups: the NEXT batch's missed
// rows are copied from host memory into a staging area (rows this update writes are flagged out beforehand), so that
// the host link's two directions work at once without depending on a second hardware queue.
template <int DTYPE, int OPT, int LPG, int ULONG, bool FETCH>
__global__ __launch_bounds__(kBlock) void k_seg_rows_long(int fetch_blocks, int long_blocks, int rows_first, int whole_runs,
                                                          const uint32_t* __restrict__ key,
                                                          const uint32_t* __restrict__ val, const int32_t* __restrict__ n_unique,
                                                          const int32_t* __restrict__ seg_start,
                                                          const int32_t* __restrict__ unique_gid,
                                                          const int32_t* __restrict__ unique_slot,
                                                          const uint32_t* __restrict__ first_bag,
                                                          const int32_t* __restrict__ chunk_run, const float* __restrict__ grad,
                                                          double* __restrict__ partial, UpdateArgs A, StageArgs F) {
    const int b = (int)blockIdx.x;
    if (FETCH && b < fetch_blocks) {   // (an instantiation of its own, so that profiles tell the two launches apart)
        __shared__ int32_t s_rbase_f[SCARS_MAX_TABLES + 1];
        stage_rows_body(b, fetch_blocks, A.meta, s_rbase_f, F);
        return;
    }
    // Workgroups start in index order.  With every row cached the long-run chunks go first (the rows' many workgroups
    // would otherwise leave them for the end); with cold rows to write the few row workgroups go first, so that the
    // host link's outward direction is busy from the start and the chunks, which need no link, run beside them
    // (one index per bag, 1.7 M lookups, 4 % of them cold: 0.90 -> 0.84 ms).
    const int rows_blocks = (int)gridDim.x - fetch_blocks - long_blocks;
    const int j = b - fetch_blocks;
    const bool is_long = rows_first ? j >= rows_blocks : j < long_blocks;
    if (is_long && whole_runs) {   // (one workgroup per chunk: long_blocks is the number of chunks)
        seg_whole_body<DTYPE, OPT, LPG, ULONG>(rows_first ? j - rows_blocks : j, val, n_unique, seg_start, unique_gid, unique_slot,
                                               chunk_run, grad, A);
    } else if (is_long) {
        seg_long_body<LPG, ULONG>(rows_first ? j - rows_blocks : j, long_blocks, key, val, n_unique, seg_start, chunk_run, grad,
                                  partial, A.D, A.Gm1, A.shift);
    } else {
        seg_rows_body<DTYPE, OPT, LPG>(rows_first ? j : j - long_blocks, rows_blocks, val, n_unique, seg_start, unique_gid,
                                       unique_slot, first_bag, grad, A);
    }
}

// Second half, in a launch of its own so that the partial sums need no fences or atomics: the group of the
// chunk in which a long run starts adds that run's partials in chunk order and applies the update.
template <int DTYPE, int OPT, int LPG>
__global__ __launch_bounds__(kBlock) void k_seg_combine(const uint32_t* __restrict__ key, const int32_t* __restrict__ n_unique,
                                                        const int32_t* __restrict__ seg_start, const int32_t* __restrict__ unique_gid,
                                                        const int32_t* __restrict__ unique_slot, const int32_t* __restrict__ chunk_run,
                                                        const double* __restrict__ partial, UpdateArgs A) {
    const int32_t* s_rbase = A.meta->row_base;   // read from the descriptor: only the few combining groups need it
    const int T = A.meta->num_tables;
    const int32_t Lv = n_unique[1];
    const int c = threadIdx.x % LPG;
    if (c * 4 >= A.D) return;
    constexpr int gpb = kBlock / LPG;
    const int64_t ngroups = (int64_t)gridDim.x * gpb;
    const int32_t nchunks = (Lv + kLongRun - 1) / kLongRun;
    for (int64_t ch = (int64_t)blockIdx.x * gpb + threadIdx.x / LPG; ch < nchunks; ch += ngroups) {
        const int32_t j0 = (int32_t)ch * kLongRun, j1 = min(j0 + kLongRun, Lv);
        if (j1 >= Lv) continue;                                  // a long run that starts here runs past j1
        const uint32_t k0 = key[j0], k1 = key[j1 - 1], kn = key[j1];
        const uint32_t kp = j0 > 0 ? key[j0 - 1] : ~k0;
        for (int side = 0; side < 2; ++side) {
            // side 0: a run that starts exactly at the chunk's first position; side 1: one that starts inside
            const bool cand = side == 0 ? (kp != k0 && kn == k0) : (k1 != k0 && kn == k1);
            if (!cand) continue;
            const int32_t r = side == 0 ? chunk_run[ch] : chunk_run[ch + 1];
            const int32_t a = seg_start[r], b = seg_start[r + 1];
            if (b - a <= kLongRun) continue;
            const uint32_t gid = (uint32_t)unique_gid[r];
            if (gid >= A.N) continue;
            RowRef<DTYPE, OPT> ref;
            ref.locate(A, s_rbase, T, (int32_t)gid, unique_slot[r]);
            float wv[4], sv[4] = {0.f, 0.f, 0.f, 0.f};
            ref.load(c, wv, sv);
            const int32_t pieces = (b - 1) / kLongRun - (int32_t)ch + 1;
            double g[4] = {0.0, 0.0, 0.0, 0.0};
            for (int32_t i = 0; i < pieces; i += kCombUnroll) {
                double2 v[kCombUnroll][2];
#pragma unroll
                for (int u = 0; u < kCombUnroll; ++u) {
                    const int32_t ii = min(i + u, pieces - 1);
                    const double2* qq = (const double2*)(partial + ((int64_t)(ch + ii) * 2 + (ii == 0 ? side : 0)) * A.D + c * 4);
                    v[u][0] = qq[0];
                    v[u][1] = qq[1];
                }
#pragma unroll
                for (int u = 0; u < kCombUnroll; ++u)
                    if (i + u < pieces) { g[0] += v[u][0].x; g[1] += v[u][0].y; g[2] += v[u][1].x; g[3] += v[u][1].y; }
            }
            ref.step_and_store(A, c, wv, sv, g);
        }
    }
}

template <int DTYPE, int OPT, int LPG>
static void launch_reduce_t(scars_handle* h, hipStream_t s, hipStream_t s2, const uint32_t* key, const uint32_t* val, const int32_t* nu,
                            const int32_t* seg_start, const int32_t* unique_gid, const float* grad, int64_t L, UpdateArgs A,
                            int fetch_blocks, StageArgs F) {
    Workspace& ws = h->ws;
    const int gpb = kBlock / LPG;
    // with cold rows to write the kernel is bound by the host link and a thousand workgroups saturate it; more only
    // take wave slots and memory queues from the kernels of the library's other streams
    // (while rows are fetched ahead beside it, few enough that the fetch gets its share of every unit's memory queue:
    // swept 128-8192 against 64-1024 workgroups of the fetch: what matters is their ratio; 128 : 384-512 and 256 : 768-1024
    // are equally good for 512-byte rows, 256 : 2048 and more for 128-byte rows; 192 : 768 is as good when nearly every
    // row of the batch is cold and better when one in five is, since the cached rows between them thin out the writes
    // of a lane group)
    const int64_t max_blocks = h->update_max_blocks > 0 ? h->update_max_blocks : (h->ahead_active ? (h->R >= 512 ? 768 : (h->R <= 128 ? 4096 : 1024)) : (h->k < h->N ? (h->R >= 512 ? 768 : 1024) : 256 * 32));
    const int rows_blocks = (int)std::max<int64_t>(1, std::min<int64_t>(div_up(L, gpb), max_blocks));
    int chunk_blocks = (int)std::max<int64_t>(1, std::min<int64_t>(div_up(div_up(L, kLongRun), gpb), 256 * 8));
    if (s2 == s && L <= h->fused_long_max_L) {
        // no table gets more than a few thousand lookups, by the caller's statement: no run is longer than that, and
        // the workgroup of the chunk a long run starts in sums all of it (no partial sums, no k_seg_combine)
        const int whole_runs = h->small_sort_applies() ? 1 : 0;
        if (whole_runs) chunk_blocks = (int)std::max<int64_t>(1, div_up(L, kLongRun));
        {
            Timed t(h, s, fetch_blocks > 0 ? "seg_rows_long+fetch_ahead" : "seg_rows_long");
            const dim3 grid(fetch_blocks + chunk_blocks + rows_blocks);
            const int rows_first = h->k < h->N ? 1 : 0;   // (rows can be cold)
#define SCARS_RL(UL, FE)                                                                                                  \
    hipLaunchKernelGGL((k_seg_rows_long<DTYPE, OPT, LPG, UL, FE>), grid, dim3(kBlock), 0, s, fetch_blocks, chunk_blocks, rows_first, whole_runs, key, \
                       val, nu, seg_start, unique_gid, ws.unique_slot, ws.first_bag, ws.chunk_run, grad, ws.partial, A, F)
            if (L <= kFusedWideMaxL) { if (fetch_blocks > 0) SCARS_RL(kTaskUnroll, true); else SCARS_RL(kTaskUnroll, false); }
            else { if (fetch_blocks > 0) SCARS_RL(kGradUnroll, true); else SCARS_RL(kGradUnroll, false); }
#undef SCARS_RL
        }
        if (whole_runs) return;
        Timed t(h, s, "seg_combine");
        hipLaunchKernelGGL((k_seg_combine<DTYPE, OPT, LPG>), dim3(chunk_blocks), dim3(kBlock), 0, s, key, nu, seg_start,
                           unique_gid, ws.unique_slot, ws.chunk_run, ws.partial, A);
        return;
    }
    {
        Timed t(h, s2, "seg_long");
        hipLaunchKernelGGL((k_seg_long<LPG>), dim3(chunk_blocks), dim3(kBlock), 0, s2, key, val, nu, seg_start, ws.chunk_run,
                           grad, ws.partial, A.D, A.Gm1, A.shift);
    }
    {
        Timed t(h, s2, "seg_combine");
        hipLaunchKernelGGL((k_seg_combine<DTYPE, OPT, LPG>), dim3(chunk_blocks), dim3(kBlock), 0, s2, key, nu, seg_start,
                           unique_gid, ws.unique_slot, ws.chunk_run, ws.partial, A);
    }
    {
        Timed t(h, s, "seg_rows");
        hipLaunchKernelGGL((k_seg_rows<DTYPE, OPT, LPG>), dim3(rows_blocks), dim3(kBlock), 0, s, val, nu, seg_start,
                           unique_gid, ws.unique_slot, ws.first_bag, grad, A);
    }
}

template <int DTYPE, int OPT>
static void launch_reduce_o(int lpg, scars_handle* h, hipStream_t s, hipStream_t s2, const uint32_t* key, const uint32_t* val,
                            const int32_t* nu, const int32_t* seg_start, const int32_t* unique_gid, const float* grad,
                            int64_t L, UpdateArgs A, int fetch_blocks, StageArgs F) {
    switch (lpg) {
#define SCARS_CASE(N) case N: launch_reduce_t<DTYPE, OPT, N>(h, s, s2, key, val, nu, seg_start, unique_gid, grad, L, A, fetch_blocks, F); break;
        SCARS_CASE(1) SCARS_CASE(2) SCARS_CASE(4) SCARS_CASE(8) SCARS_CASE(16) SCARS_CASE(32) SCARS_CASE(64)
        SCARS_CASE(128)
#undef SCARS_CASE
    }
}

template <int DTYPE, int OPT>
static void launch_small_update_o(int lpg, scars_handle* h, hipStream_t s, const uint32_t* key, const uint32_t* val,
                                  const float* grad, int64_t L, const UpdateArgs& A) {
    Timed t(h, s, "small_update");
    const int long_blocks = (int)div_up(L, kLongRun);
    switch (lpg) {
#define SCARS_CASE(N)                                                                                                      \
    case N: {                                                                                                              \
        const int rows_blocks = (int)std::max<int64_t>(1, std::min<int64_t>(div_up(L, kBlock / N), 256 * 32));            \
        hipLaunchKernelGGL((k_small_update<DTYPE, OPT, N>), dim3(long_blocks + rows_blocks), dim3(kBlock), 0, s, long_blocks, \
                           (int32_t)L, h->buf.max_L, key, val, h->ws.seg_start, h->ws.unique_slot, grad, A);               \
    } break;
        SCARS_CASE(1) SCARS_CASE(2) SCARS_CASE(4) SCARS_CASE(8) SCARS_CASE(16) SCARS_CASE(32) SCARS_CASE(64)
        SCARS_CASE(128)
#undef SCARS_CASE
    }
}

static void launch_small_update(scars_handle* h, hipStream_t s, const uint32_t* key, const uint32_t* val, const float* grad,
                                int64_t L, const UpdateArgs& A) {
    const int lpg = next_pow2_host(h->D / 4);
    if (h->dtype == SCARS_DTYPE_F32) {
        if (h->optimizer == SCARS_OPT_SGD) launch_small_update_o<SCARS_DTYPE_F32, SCARS_OPT_SGD>(lpg, h, s, key, val, grad, L, A);
        else launch_small_update_o<SCARS_DTYPE_F32, SCARS_OPT_ADAGRAD>(lpg, h, s, key, val, grad, L, A);
    } else {
        if (h->optimizer == SCARS_OPT_SGD) launch_small_update_o<SCARS_DTYPE_BF16, SCARS_OPT_SGD>(lpg, h, s, key, val, grad, L, A);
        else launch_small_update_o<SCARS_DTYPE_BF16, SCARS_OPT_ADAGRAD>(lpg, h, s, key, val, grad, L, A);
    }
}

// Integer half of the backward pass: (gid, bag) pairs, their sort, the run starts.  It depends on the remap outputs
// only, not on the gradient, so it may run on another stream while the forward pass runs.  `staged`: cold rows take
// their current value from the staging area (the forward pass of the same batch fills it).
hipError_t launch_bwd_segments(scars_handle* h, hipStream_t s, const int32_t* off, int64_t L, int64_t B,
                               const scars_remap_out* rm, bool staged, const scars_bwd_out* out, int* res_out,
                               bool* by_position) {
    Workspace& ws = h->ws;
    int32_t* n_unique = out ? out->n_unique : ws.n_unique;
    int32_t* seg_start = out ? out->seg_start : ws.seg_start;
    int32_t* unique_gid = out ? out->unique_gid : ws.unique_gid;
    const int64_t G = (int64_t)h->T * B;
    // the remap of this batch may have left the pairs in the first sort buffer; the sort below uses them up
    const bool have_pairs = h->pairs_valid && h->pairs_gid == rm->gid && h->pairs_off == off && h->pairs_L == L && h->pairs_B == B;
    h->pairs_valid = false;
    // ... and its forward pass may already have sorted each table's piece (beside the fetch of the missed rows)
    const bool small = h->small_sort_applies();
    const bool pieces_sorted = small && h->small_sorted && h->small_gid == rm->gid && h->small_off == off &&
                               h->small_L == L && h->small_B == B;
    h->small_sorted = false;
    if (!have_pairs && !pieces_sorted) {
        Timed t(h, s, "bwd_pairs");
        const int lpb = pairs_lanes_per_bag(L, G);
        hipLaunchKernelGGL(k_bwd_pairs, dim3((unsigned)div_up(G * lpb, kBlock)), dim3(kBlock), 0, s, rm->gid, off,
                           (int32_t)L, G, lpb, bag_shift_host(G), ws.key_buf[0], ws.val_buf[0]);
    }
    int bits = 1;
    while (bits < 32 && ((int64_t)1 << bits) <= h->N) ++bits;   // 2^bits - 1 >= N: the sentinel stays the largest key
    int res = 0;
    // the caller has stated that no table gets more than a few thousand lookups: each table's piece is sorted in LDS
    if (small) {
        const int limit = (int)h->table_lookups_limit;
        // the caller of this function can update by position (no list of runs wanted): the sort leaves what that needs
        bool runs = by_position != nullptr;
        if (!pieces_sorted) {
            const SmallRunArgs run = small_run_args(h, rm, staged);
            hipError_t e = launch_small_sort(h, s, ws.key_buf, ws.val_buf, off, L, B, runs ? &run : nullptr);
            if (e != hipSuccess) return e;
        } else {
            ++h->n_small_sorted_used;
            runs = runs && h->small_runs && h->small_runs_staged == staged;
        }
        if (runs) {      // the sorted pieces stay where they are
            *res_out = 1;
            *by_position = true;
            return hipGetLastError();
        }
        *res_out = 0;
        Timed t(h, s, "small_segments");
        hipLaunchKernelGGL(k_small_segments, dim3(h->T), dim3(kBlock), 0, s, ws.key_buf[1], ws.val_buf[1], off, B, (int32_t)L,
                           h->T, limit, ws.sort_hist, ws.sort_hist + h->T, ws.key_buf[0], ws.val_buf[0], n_unique, seg_start,
                           unique_gid, out ? out->sorted_gid : nullptr, out ? out->sorted_bag : nullptr, ws.chunk_run,
                           h->buf.slot_of, (uint32_t)h->N, ws.unique_slot, ws.first_bag, G, rm->gid, rm->loc, (int32_t)h->k,
                           staged ? 1 : 0, bag_shift_host(G), L <= kSegViaLocMaxL ? 1 : 0);
        return hipGetLastError();
    }
    hipError_t e = launch_radix_sort_pairs(h, s, ws.key_buf, ws.val_buf, L, nullptr, bits, &res);
    if (e != hipSuccess) return e;
    *res_out = res;
    const uint32_t* key = ws.key_buf[res];
    const uint32_t* val = ws.val_buf[res];
    const int nb = (int)div_up(L, kScanTile);
    {
        Timed t(h, s, "seg_count");
        hipLaunchKernelGGL(k_seg_count, dim3(nb), dim3(kBlock), 0, s, key, L, ws.blk_seg_a, ws.blk_seg_b);
    }
    const bool scan = nb > h->fused_scan_max_tiles;   // few tiles: the writer adds up the tile counts itself
    if (scan) {
        Timed t(h, s, "seg_scan");
        hipLaunchKernelGGL(k_seg_scan, dim3(1), dim3(kBlock), 0, s, ws.blk_seg_a, ws.blk_seg_b, nb, n_unique);
    }
    {
        Timed t(h, s, "seg_write");
        hipLaunchKernelGGL(k_seg_write, dim3(nb), dim3(kBlock), 0, s, key, val, L, ws.blk_seg_a, ws.blk_seg_b, scan ? 1 : 0,
                           n_unique, seg_start, unique_gid, out ? out->sorted_gid : nullptr, out ? out->sorted_bag : nullptr,
                           ws.chunk_run, h->buf.slot_of, (uint32_t)h->N, ws.unique_slot, ws.first_bag, off, G, rm->gid,
                           rm->loc, (int32_t)h->k, staged ? 1 : 0, bag_shift_host(G), L <= kSegViaLocMaxL ? 1 : 0);
    }
    return hipGetLastError();
}

hipError_t launch_bwd(scars_handle* h, hipStream_t s, const int32_t* off, int64_t L, int64_t B,
                      const scars_remap_out* rm, const float* grad, float lr, float eps, const scars_bwd_out* out,
                      const scars_remap_out* next_rm, const int32_t* next_off, int64_t next_L, int64_t next_B) {
    Workspace& ws = h->ws;
    // rows fetched by this batch's forward pass are still in a staging area: cold rows are read from there
    const int area = h->staged_area(rm->loc);
    const bool use_staged = area >= 0;
    h->stg[0].valid = h->stg[1].valid = false;   // this call changes the rows
    h->ahead.valid = false;                      // ... also rows fetched ahead beside an earlier update
    int32_t* n_unique = out ? out->n_unique : ws.n_unique;
    int32_t* seg_start = out ? out->seg_start : ws.seg_start;
    int32_t* unique_gid = out ? out->unique_gid : ws.unique_gid;
    const int64_t G = (int64_t)h->T * B;
    // segments prepared on the side stream for this very batch, by its remap or (look-ahead) beside the previous
    // batch's update (the caller's stream has already been made to wait for them); they are in the workspace arrays,
    // built for staged cold rows when misses are possible
    const bool prepared = h->presort_valid && h->presort_gid == rm->gid && h->presort_loc == rm->loc &&
                          h->presort_off == off && h->presort_L == L && h->presort_B == B && !out &&
                          h->presort_staged == use_staged;
    h->presort_valid = false;
    if (prepared || L == 0) h->small_sorted = false;   // (otherwise launch_bwd_segments below takes it or drops it)
    if (L == 0) {
        Timed t(h, s, "bwd_empty");
        hipLaunchKernelGGL(k_bwd_empty, dim3(1), dim3(kWave), 0, s, n_unique, seg_start);
        return hipGetLastError();
    }
    int res = h->presort_res;
    if (prepared) ++h->n_prepared_used;
    bool by_position = false;
    if (!prepared) {
        // (a caller who wants the sorted segments, or the look-ahead order, whose fetch leaves out this batch's distinct
        // rows, needs the list of runs)
        const bool can_go_by_position = !out && !next_rm && !h->lookahead;
        hipError_t e = launch_bwd_segments(h, s, off, L, B, rm, use_staged, out, &res, can_go_by_position ? &by_position : nullptr);
        if (e != hipSuccess) return e;
    }
    const uint32_t* key = ws.key_buf[res];
    const uint32_t* val = ws.val_buf[res];
    UpdateArgs A{ws.meta, h->buf.slot_of, h->buf.cache, h->buf.state_cache, lr, eps, h->D,
                 use_staged ? ws.staging[area] : nullptr, (int32_t)h->k, (uint32_t)h->N,
                 (uint32_t)std::max<int64_t>(G - 1, 0), bag_shift_host(G)};
    if (by_position) {
        h->ahead_active = false;
        const hipError_t e = pf_join(h, s);   // (a fetch still running beside an earlier update reads host rows)
        if (e != hipSuccess) return e;
        launch_small_update(h, s, key, val, grad, L, A);
        return hipGetLastError();
    }
    // Look-ahead.  (1) The integer half of the next batch's backward pass is prepared beside this update, on the side
    // stream and in the second set of segment arrays (this update still reads the first); the sets change places once
    // the update kernels are enqueued.  It is enqueued before the fetch: should the two library streams share a
    // hardware queue, a fetch of milliseconds in front of it would push it beside the next forward pass.
    const bool fetch_next = next_rm && next_L > 0 && h->k < h->N;
    // (also when every row is cached and nothing is fetched: the sort of a batch is a chain of short launches that
    // hides behind an update several times as long: multi_hot 0.358 -> 0.311 ms per step, uniform ids 0.70 -> 0.66)
    const bool prep_next = next_rm && next_L > 0 && h->presort_min_L > 0 && next_L >= h->presort_min_L;
    if (prep_next) {
        swap_segment_sets(h);
        const hipError_t e = start_presort(h, s, next_off, next_L, next_B, next_rm);
        swap_segment_sets(h);
        if (e != hipSuccess) return e;
    }
    // (2) The next batch's missed rows, except those this update writes, are fetched while it runs (a stream and a
    // staging area of their own); the list of this batch's distinct rows is complete at this point of stream s.
    h->ahead_active = false;
    {   // a fetch still running beside an earlier update reads host rows: it must be over before this update writes any
        const hipError_t e = pf_join(h, s);
        if (e != hipSuccess) return e;
    }
    const int lpg = next_pow2_host(h->D / 4);
    // long runs (HBM-bound) beside the per-row kernel (bound by the host link while rows are cold)
    hipStream_t s2 = s;
    const bool split = !prep_next && h->presort_min_L > 0 && L >= h->presort_min_L && h->k < h->N;
    // the fetch rides in the update's own launch whenever long runs and rows share one (no second hardware queue
    // needed for the two directions of the link to overlap); otherwise it goes to the library's second stream
    const bool fuse_fetch = fetch_next && h->fused_fetch && !split && L <= h->fused_long_max_L;
    StageArgs F{};
    int fetch_blocks = 0;
    h->timer_tag = (fetch_next && !fuse_fetch) ? ++h->timer_serial : 0;
    if (fetch_next) {
        hipError_t e = launch_fetch_ahead(h, s, next_rm, next_L, unique_gid, n_unique, use_staged ? 1 - area : 0,
                                          fuse_fetch ? &F : nullptr, &fetch_blocks);
        if (e != hipSuccess) return e;
        if (!fuse_fetch) fetch_blocks = 0;
        h->ahead_active = true;
    }
    if (split) {
        hipError_t e = side_fork(h, s);
        if (e != hipSuccess) return e;
        s2 = h->side;
    }
    if (h->dtype == SCARS_DTYPE_F32) {
        if (h->optimizer == SCARS_OPT_SGD) launch_reduce_o<SCARS_DTYPE_F32, SCARS_OPT_SGD>(lpg, h, s, s2, key, val, n_unique, seg_start, unique_gid, grad, L, A, fetch_blocks, F);
        else launch_reduce_o<SCARS_DTYPE_F32, SCARS_OPT_ADAGRAD>(lpg, h, s, s2, key, val, n_unique, seg_start, unique_gid, grad, L, A, fetch_blocks, F);
    } else {
        if (h->optimizer == SCARS_OPT_SGD) launch_reduce_o<SCARS_DTYPE_BF16, SCARS_OPT_SGD>(lpg, h, s, s2, key, val, n_unique, seg_start, unique_gid, grad, L, A, fetch_blocks, F);
        else launch_reduce_o<SCARS_DTYPE_BF16, SCARS_OPT_ADAGRAD>(lpg, h, s, s2, key, val, n_unique, seg_start, unique_gid, grad, L, A, fetch_blocks, F);
    }
    if (split) {
        hipError_t e = hipEventRecord(h->ev_join, h->side);
        if (e == hipSuccess) e = hipStreamWaitEvent(s, h->ev_join, 0);
        if (e != hipSuccess) return e;
    }
    h->timer_tag = 0;
    if (prep_next) swap_segment_sets(h);   // what was prepared is what the next call finds
    return hipGetLastError();
}

}  // namespace scars
