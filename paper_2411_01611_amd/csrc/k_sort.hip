// Stable LSD radix sort of (uint32 key, uint32 value) pairs, up to 9 bits per pass, staged through LDS.
//
// Used for (a) ordering the selected hot rows by descending count (key = ~count, value = gid; the input is
// in ascending gid order, so stability gives "lower id first among equal counts"), and (b) ordering a
// batch's lookups by (gid, position) for the backward pass (key = gid, value = bag; the input is in
// position order).  Per pass: per-tile digit histogram (one row of `bins` counts per tile) -> per-digit exclusive scan
// down the tiles (eight digit columns per workgroup, so that a row of lanes touches one 32-byte piece of a tile's row) -> scatter
// in which each tile is first ordered in LDS (wave-level multi-split; equal digits are matched through LDS) and then written
// out as contiguous runs per digit.  The number of passes is ceil(bits / 9) and the digit width is
// ceil(bits / passes), so 26-bit row ids take three 9-bit passes instead of four 8-bit ones.
#include "scars_dev.h"

namespace scars {

constexpr int kMaxBins = kSortMaxBins;
constexpr int kWaves = kBlock / kWave;

// hist is tile-major: hist[tile * bins + d].  Each wave counts into a histogram of its own in LDS (one atomic per key;
// matching the lanes that hold equal digits first, as the scatter kernel does for its ranks, cost twice the time it
// saved: nine ballots per key against a conflict now and then).  Keys are read 16 bytes per lane.
template <int ROUNDS>
__global__ __launch_bounds__(kBlock) void k_sort_hist(const uint32_t* __restrict__ keys, int64_t n, const int32_t* __restrict__ d_n,
                                                      int shift, int dbits, uint32_t* __restrict__ hist, int nb) {
    __shared__ uint32_t s_hist[kWaves * kMaxBins];
    static_assert(ROUNDS % 4 == 0, "a lane takes four consecutive keys per load");
    if (d_n) n = min(n, (int64_t)max(*d_n, 0));    // the pair count may live on the device (n is then its bound)
    const int bins = 1 << dbits;
    const uint32_t mask = (uint32_t)bins - 1u;
    for (int i = threadIdx.x; i < kWaves * kMaxBins; i += kBlock) s_hist[i] = 0;
    __syncthreads();
    uint32_t* wh = s_hist + wave_id() * kMaxBins;
    const int64_t tile0 = (int64_t)blockIdx.x * (kBlock * ROUNDS);
    uint32_t kk[ROUNDS];
#pragma unroll
    for (int q = 0; q < ROUNDS / 4; ++q) {
        const int64_t i = tile0 + ((int64_t)q * kBlock + threadIdx.x) * 4;
        if (i + 3 < n) {
            const uint4 v = *(const uint4*)(keys + i);           // tile0 and i are multiples of 4: 16-byte aligned
            kk[4 * q] = v.x; kk[4 * q + 1] = v.y; kk[4 * q + 2] = v.z; kk[4 * q + 3] = v.w;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) kk[4 * q + e] = i + e < n ? keys[i + e] : 0u;
        }
    }
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) {
        const int64_t i = tile0 + ((int64_t)(r / 4) * kBlock + threadIdx.x) * 4 + (r % 4);
        const bool valid = i < n;
        const uint32_t d = (kk[r] >> shift) & mask;
        if (valid) atomicAdd(&wh[d], 1u);
    }
    __syncthreads();
    for (int d = threadIdx.x; d < bins; d += kBlock) {
        uint32_t c = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) c += s_hist[w * kMaxBins + d];
        hist[(int64_t)blockIdx.x * bins + d] = c;
    }
}

// Exclusive scan of every digit's counts down the tiles, in place; digit totals to tot[digit].  A workgroup takes a
// group of g = min(kScanDigits, bins) neighbouring digits; lane (row, dg) = (tid / g, tid % g) owns the digit's counts
// of `per` consecutive tiles.  Three steps whatever the number of tiles: every lane adds up its tiles (independent
// loads), one scan of those sums across the rows of lanes, then every lane writes the running sums of its tiles.
constexpr int kScanDigits = 8;  // digits per workgroup (fewer when a pass has fewer bins): 32-byte pieces of a tile's row; swept 1/2/4/8
constexpr int kScanUnroll = 16;  // loads in flight per lane: the kernel is a chain of round trips, not of bytes
__global__ __launch_bounds__(kBlock) void k_sort_scan(uint32_t* __restrict__ hist, int nb, int bins, int g,
                                                      uint32_t* __restrict__ tot) {
    __shared__ uint32_t s_w[kWaves][kScanDigits];
    const int dg = threadIdx.x % g, row = threadIdx.x / g;
    const int rows = kBlock / g;                 // rows of lanes in the workgroup
    const int d = blockIdx.x * g + dg;
    const int per = (nb + rows - 1) / rows;
    const int t0 = min(row * per, nb), t1 = min(t0 + per, nb);
    uint32_t* const col = hist + d;
    uint32_t sum = 0;
    for (int t = t0; t < t1; t += kScanUnroll) {
        uint32_t v[kScanUnroll];
#pragma unroll
        for (int i = 0; i < kScanUnroll; ++i) v[i] = t + i < t1 ? col[(int64_t)(t + i) * bins] : 0u;
#pragma unroll
        for (int i = 0; i < kScanUnroll; ++i) sum += v[i];
    }
    // inclusive scan of `sum` over the rows of this wave (lanes of one digit are g apart), then over the waves
    uint32_t inc = sum;
    for (int st = g; st < kWave; st <<= 1) {
        const uint32_t o = __shfl_up(inc, st, kWave);
        if (lane_id() >= st) inc += o;
    }
    if (lane_id() >= kWave - g) s_w[wave_id()][dg] = inc;    // the wave's last row holds the wave's total
    __syncthreads();
    uint32_t run = inc - sum, all = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const uint32_t t = s_w[w][dg];
        if (w < wave_id()) run += t;
        all += t;
    }
    for (int t = t0; t < t1; t += kScanUnroll) {
        uint32_t v[kScanUnroll];
#pragma unroll
        for (int i = 0; i < kScanUnroll; ++i) v[i] = t + i < t1 ? col[(int64_t)(t + i) * bins] : 0u;
#pragma unroll
        for (int i = 0; i < kScanUnroll; ++i) {
            if (t + i < t1) col[(int64_t)(t + i) * bins] = run;
            run += v[i];
        }
    }
    if (row == 0) tot[d] = all;
}

// The same with a lane's counts kept in registers between the two sweeps (no second read of the column, every load
// of the first sweep in flight at once): for up to PER tiles per lane; the host picks, and takes the kernel above
// beyond 40 (4.3 M pairs, 33 tiles per lane: 11.7 -> 9.4 us between events; 655 k pairs, 10 per lane: unchanged).
template <int PER>
__global__ __launch_bounds__(kBlock) void k_sort_scan_reg(uint32_t* __restrict__ hist, int nb, int bins, int g,
                                                          uint32_t* __restrict__ tot) {
    __shared__ uint32_t s_w[kWaves][kScanDigits];
    const int dg = threadIdx.x % g, row = threadIdx.x / g;
    const int rows = kBlock / g;
    const int d = blockIdx.x * g + dg;
    const int per = (nb + rows - 1) / rows;      // <= PER (checked by the host)
    const int t0 = min(row * per, nb), t1 = min(t0 + per, nb);
    uint32_t* const col = hist + d;
    uint32_t v[PER];
    uint32_t sum = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) v[i] = t0 + i < t1 ? col[(int64_t)(t0 + i) * bins] : 0u;
#pragma unroll
    for (int i = 0; i < PER; ++i) sum += v[i];
    uint32_t inc = sum;
    for (int st = g; st < kWave; st <<= 1) {
        const uint32_t o = __shfl_up(inc, st, kWave);
        if (lane_id() >= st) inc += o;
    }
    if (lane_id() >= kWave - g) s_w[wave_id()][dg] = inc;
    __syncthreads();
    uint32_t run = inc - sum, all = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const uint32_t t = s_w[w][dg];
        if (w < wave_id()) run += t;
        all += t;
    }
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        if (t0 + i < t1) col[(int64_t)(t0 + i) * bins] = run;
        run += v[i];
    }
    if (row == 0) tot[d] = all;
}

// Tile = 256 * ROUNDS pairs; wave w owns the contiguous quarter [w * 64 * ROUNDS, ...) in ROUNDS rounds of 64.
template <int ROUNDS>
__global__ __launch_bounds__(kBlock) void k_sort_scatter(const uint32_t* __restrict__ kin, const uint32_t* __restrict__ vin,
                                                         uint32_t* __restrict__ kout, uint32_t* __restrict__ vout,
                                                         int64_t n, const int32_t* __restrict__ d_n, int shift, int dbits,
                                                         const uint32_t* __restrict__ hist, const uint32_t* __restrict__ tot, int nb) {
    constexpr int kTile = kBlock * ROUNDS;
    if (d_n) n = min(n, (int64_t)max(*d_n, 0));
    // Workgroups are handed to the chip's eight dies (each with an L2 of its own) in turn; tiles next to each other
    // write next to each other (the runs of one digit from consecutive tiles are adjacent in the output), so each
    // die takes a contiguous eighth of the tiles and its L2 can put the pieces of a line together before writing it.
    const int per_die = (nb + 7) / 8;
    const int tile = (int)(blockIdx.x % 8) * per_die + (int)(blockIdx.x / 8);
    if (tile >= nb || (int64_t)tile * kTile >= n) return;   // whole workgroup: nothing of this tile is in use
    constexpr int kPerWave = kWave * ROUNDS;
    // the ordered tile; before that the same memory holds, per wave and digit, the lanes of the round in hand
    constexpr int kPairWords = 2 * kTile > 2 * kWaves * kMaxBins ? 2 * kTile : 2 * kWaves * kMaxBins;
    __shared__ __align__(8) uint32_t s_pairs[kPairWords];
    uint32_t* const s_key = s_pairs;
    uint32_t* const s_val = s_pairs + kTile;
    __shared__ uint32_t s_wh[kWaves * kMaxBins];   // per-wave digit counters, then exclusive wave bases
    __shared__ uint32_t s_dstart[kMaxBins];         // first LDS position of each digit in this tile
    __shared__ uint32_t s_goff[kMaxBins];           // global position of this tile's first pair of each digit
    __shared__ uint32_t s_scan[8];

    const int tid = threadIdx.x, lane = lane_id(), w = wave_id();
    const int bins = 1 << dbits;
    const uint32_t mask = (uint32_t)bins - 1u;
    const int64_t tile0 = (int64_t)tile * kTile;
    const int tile_n = (int)min((int64_t)kTile, n - tile0);

    // the tile's pairs are requested first, so that their round trip overlaps the one of the digit offsets below
    uint32_t key[ROUNDS], val[ROUNDS], loc[ROUNDS];
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) {
        const int p = w * kPerWave + r * kWave + lane;          // position inside the tile
        const bool valid = p < tile_n;
        key[r] = valid ? kin[tile0 + p] : 0xFFFFFFFFu;
        val[r] = valid ? vin[tile0 + p] : 0u;
    }
    for (int i = tid; i < kWaves * kMaxBins; i += kBlock) s_wh[i] = 0;
    for (int i = tid; i < 2 * kWaves * kMaxBins; i += kBlock) s_pairs[i] = 0;
    {   // global base of every digit = scan of the digit totals, plus this tile's offset inside the digit
        uint32_t carry = 0;
        for (int base = 0; base < bins; base += kBlock) {
            const int d = base + tid;
            const uint32_t v = d < bins ? tot[d] : 0u;
            uint32_t total;
            const uint32_t ex = block_exclusive_scan(v, s_scan, &total);
            if (d < bins) s_goff[d] = carry + ex + hist[(int64_t)tile * bins + d];
            carry += total;
        }
    }
    __syncthreads();

    // Stable rank of every pair among its wave's pairs of the same digit.  The lanes of a round that share a digit are
    // matched; the first lane of each such set adds the set's size to the wave's counter of the digit and gets back
    // what was there (the sets of a round have distinct digits); every lane then takes that number from its set's
    // first lane and adds its own place in the set.
    uint32_t* wh = s_wh + w * kMaxBins;
    uint32_t old[ROUNDS];
    int lead[ROUNDS];
    // the lanes sharing a digit are found through LDS instead of nine ballots: every lane sets its bit in the
    // wave's 64-bit word of its digit, then reads the word back (one wave's LDS operations are carried out in
    // order, and all lanes of an instruction before the next); the set's first lane clears the word again
    unsigned long long* const mk = (unsigned long long*)s_pairs + w * kMaxBins;
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) {
        const int p = w * kPerWave + r * kWave + lane;
        const bool valid = p < tile_n;
        const uint32_t d = (key[r] >> shift) & mask;
        if (valid) atomicOr(&mk[d], 1ull << lane);
        __builtin_amdgcn_wave_barrier();
        const uint64_t m = valid ? *(volatile unsigned long long*)&mk[d] : (1ull << lane);
        __builtin_amdgcn_wave_barrier();
        const int rk = rank_below(m);
        lead[r] = __ffsll((unsigned long long)m) - 1;
        loc[r] = (uint32_t)rk;
        old[r] = 0u;
        if (valid && rk == 0) {
            *(volatile unsigned long long*)&mk[d] = 0ull;
            old[r] = atomicAdd(&wh[d], (uint32_t)__popcll(m));
        }
        __builtin_amdgcn_wave_barrier();
    }
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) loc[r] += __shfl(old[r], lead[r], kWave);   // stable rank among this wave's pairs of digit d
    __syncthreads();
    {   // per digit: wave counts -> exclusive wave bases; tile count of the digit -> LDS start of the digit
        uint32_t carry = 0;
        for (int base = 0; base < bins; base += kBlock) {
            const int d = base + tid;
            uint32_t run = 0;
            if (d < bins) {
#pragma unroll
                for (int ww = 0; ww < kWaves; ++ww) {
                    const uint32_t t = s_wh[ww * kMaxBins + d];
                    s_wh[ww * kMaxBins + d] = run;
                    run += t;
                }
            }
            uint32_t total;
            const uint32_t ex = block_exclusive_scan(run, s_scan, &total);
            if (d < bins) s_dstart[d] = carry + ex;
            carry += total;
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) {
        const int p = w * kPerWave + r * kWave + lane;
        if (p < tile_n) {
            const uint32_t d = (key[r] >> shift) & mask;
            const uint32_t q = s_dstart[d] + s_wh[w * kMaxBins + d] + loc[r];
            s_key[q] = key[r];
            s_val[q] = val[r];
        }
    }
    __syncthreads();
    for (int q = tid; q < tile_n; q += kBlock) {
        const uint32_t k = s_key[q];
        const uint32_t d = (k >> shift) & mask;
        const uint32_t dst = s_goff[d] + ((uint32_t)q - s_dstart[d]);
        kout[dst] = k;
        vout[dst] = s_val[q];
    }
}

// ---- small batches: one workgroup sorts one table's pairs entirely in LDS ------------------------------------------
// A batch is table-major, so the pairs of table t sit at positions [offsets[t*B], offsets[(t+1)*B]) and their keys lie
// in the table's own range of row ids: sorting each table's piece by itself sorts the whole array.  When the caller
// has stated that no table gets more than kSmallSortCap lookups per batch (one index per sample and table with a batch of
// a few thousand samples is the case), a workgroup per table does all the passes of its piece in LDS, on keys made
// table-local (a table of a thousand rows takes two passes, not three), in one launch instead of three per pass.
// Invalid lookups (key 0xFFFFFFFF) come last in the whole array, as in the general sort: the workgroups write their
// sorted pieces in place and each piece's numbers of valid pairs and of distinct rows; the launch that lists the run
// starts (k_small_segments) moves the pieces to where the counts of the tables before them put them (every piece
// stays where it is when no lookup is invalid).
static_assert(kSmallSortCap % kBlock == 0, "a table's piece is dealt out in whole rounds of the workgroup");

__global__ __launch_bounds__(kBlock) void k_small_sort(const Meta* __restrict__ meta, SmallSortArgs S) {
    small_sort_body((int)blockIdx.x, meta, S);
}

// The pairs are in key[0] / val[0] (position order); each table's sorted piece is left at the piece's own place in
// key[1] / val[1], the tables' counts of valid pairs and of distinct rows in the first 2 T words of the sort's count matrix.
hipError_t launch_small_sort(scars_handle* h, hipStream_t s, uint32_t* key[2], uint32_t* val[2], const int32_t* off,
                             int64_t L, int64_t B, const SmallRunArgs* run) {
    Timed t(h, s, "small_sort");
    SmallSortArgs Q = small_sort_args(h, key, val, off, L, B);
    if (run) Q.run = *run;
    hipLaunchKernelGGL(k_small_sort, dim3(h->T), dim3(kBlock), 0, s, h->ws.meta, Q);
    return hipGetLastError();
}

template <int ROUNDS>
static void sort_passes(scars_handle* h, hipStream_t s, uint32_t* key[2], uint32_t* val[2], int64_t n, const int32_t* d_n,
                        int bits, int* cur) {
    const int nb = (int)div_up(n, kBlock * ROUNDS);
    const int passes = (int)div_up(bits, 9);
    const int dbits = (int)div_up(bits, passes);
    for (int p = 0; p < passes; ++p) {
        const int shift = p * dbits;
        {
            Timed t(h, s, "sort_hist");
            hipLaunchKernelGGL((k_sort_hist<ROUNDS>), dim3(nb), dim3(kBlock), 0, s, key[*cur], n, d_n, shift, dbits,
                               h->ws.sort_hist, nb);
        }
        {
            Timed t(h, s, "sort_scan");
            const int bins = 1 << dbits, g = std::min(kScanDigits, bins);
            const int per = (int)div_up(nb, kBlock / g);     // tiles per lane
            if (per <= 16)
                hipLaunchKernelGGL((k_sort_scan_reg<16>), dim3(bins / g), dim3(kBlock), 0, s, h->ws.sort_hist, nb, bins, g, h->ws.sort_tot);
            else if (per <= 40)
                hipLaunchKernelGGL((k_sort_scan_reg<40>), dim3(bins / g), dim3(kBlock), 0, s, h->ws.sort_hist, nb, bins, g, h->ws.sort_tot);
            else
                hipLaunchKernelGGL(k_sort_scan, dim3(bins / g), dim3(kBlock), 0, s, h->ws.sort_hist, nb, bins, g, h->ws.sort_tot);
        }
        {
            Timed t(h, s, "sort_scatter");
            hipLaunchKernelGGL((k_sort_scatter<ROUNDS>), dim3((nb + 7) / 8 * 8), dim3(kBlock), 0, s, key[*cur], val[*cur], key[*cur ^ 1],
                               val[*cur ^ 1], n, d_n, shift, dbits, h->ws.sort_hist, h->ws.sort_tot, nb);
        }
        *cur ^= 1;
    }
}

hipError_t launch_radix_sort_pairs(scars_handle* h, hipStream_t s, uint32_t* key[2], uint32_t* val[2], int64_t n,
                                   const int32_t* d_n, int bits, int* result_buffer) {
    int cur = 0;
    if (n > 0) {
        // small inputs: small tiles, so that there are enough workgroups to fill the chip (measured: 655 k pairs are
        // fastest with tiles of 2048, 4.3 M pairs with tiles of 4096)
        if (n <= ((int64_t)1 << 18)) sort_passes<kSortRoundsSmall>(h, s, key, val, n, d_n, bits, &cur);
        else if (n < ((int64_t)1 << 22)) sort_passes<kSortRoundsMid>(h, s, key, val, n, d_n, bits, &cur);
        else sort_passes<kSortRoundsLarge>(h, s, key, val, n, d_n, bits, &cur);
    }
    *result_buffer = cur;
    return hipGetLastError();
}

}  // namespace scars
