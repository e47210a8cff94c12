// Stable LSD radix sort of (uint32 key, uint32 value) pairs, up to 9 bits per pass, staged through LDS.
//
// Used for (a) ordering the selected hot rows by descending count (key = ~count, value = gid; the input is
// in ascending gid order, so stability gives "lower id first among equal counts"), and (b) ordering a
// batch's lookups by (gid, position) for the backward pass (key = gid, value = bag; the input is in
// position order).  Per pass: per-tile digit histogram -> per-digit exclusive scan over tiles -> scatter
// in which each tile is first ordered in LDS (wave-level multi-split by ballot matching) and then written
// out as contiguous runs per digit.  The number of passes is ceil(bits / 9) and the digit width is
// ceil(bits / passes), so 26-bit row ids take three 9-bit passes instead of four 8-bit ones.
#include "scars_dev.h"

namespace scars {

constexpr int kMaxBins = kSortMaxBins;
constexpr int kWaves = kBlock / kWave;

// Lanes of the wave that hold the same digit as this lane (valid lanes only): one ballot per digit bit.
__device__ __forceinline__ uint64_t match_digit(uint32_t d, bool valid, int dbits) {
    uint64_t m = ballot64(valid);
    for (int b = 0; b < dbits; ++b) {
        const bool bit = (d >> b) & 1u;
        const uint64_t bal = ballot64(bit);
        m &= bit ? bal : ~bal;
    }
    return m;
}

// hist is digit-major: hist[d * nb + tile].  Each wave counts into a histogram of its own; lanes holding the same
// digit are matched by ballots and only the first of them adds their number (equal keys, which skewed row ids have
// many of, then cost one LDS operation instead of one each).  Keys are read 16 bytes per lane.
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
        const uint64_t m = match_digit(d, valid, dbits);
        if (valid && rank_below(m) == 0) atomicAdd(&wh[d], (uint32_t)__popcll(m));   // distinct digits: distinct words
    }
    __syncthreads();
    for (int d = threadIdx.x; d < bins; d += kBlock) {
        uint32_t c = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) c += s_hist[w * kMaxBins + d];
        hist[(int64_t)d * nb + blockIdx.x] = c;
    }
}

// One workgroup per digit: exclusive scan of that digit's per-tile counts, digit total to tot[digit].
__global__ __launch_bounds__(kBlock) void k_sort_scan(uint32_t* __restrict__ hist, int nb, uint32_t* __restrict__ tot) {
    __shared__ uint32_t s_scan[8];
    uint32_t* row = hist + (int64_t)blockIdx.x * nb;
    uint32_t carry = 0;
    for (int base = 0; base < nb; base += kBlock) {
        const int i = base + threadIdx.x;
        const uint32_t v = i < nb ? row[i] : 0u;
        uint32_t total;
        const uint32_t ex = block_exclusive_scan(v, s_scan, &total);
        if (i < nb) row[i] = carry + ex;
        carry += total;
    }
    if (threadIdx.x == 0) tot[blockIdx.x] = carry;
}

// Tile = 256 * ROUNDS pairs; wave w owns the contiguous quarter [w * 64 * ROUNDS, ...) in ROUNDS rounds of 64.
template <int ROUNDS>
__global__ __launch_bounds__(kBlock) void k_sort_scatter(const uint32_t* __restrict__ kin, const uint32_t* __restrict__ vin,
                                                         uint32_t* __restrict__ kout, uint32_t* __restrict__ vout,
                                                         int64_t n, const int32_t* __restrict__ d_n, int shift, int dbits,
                                                         const uint32_t* __restrict__ hist, const uint32_t* __restrict__ tot, int nb) {
    constexpr int kTile = kBlock * ROUNDS;
    if (d_n) n = min(n, (int64_t)max(*d_n, 0));
    if ((int64_t)blockIdx.x * kTile >= n) return;   // whole workgroup: nothing of this tile is in use
    constexpr int kPerWave = kWave * ROUNDS;
    __shared__ uint32_t s_key[kTile];
    __shared__ uint32_t s_val[kTile];
    __shared__ uint32_t s_wh[kWaves * kMaxBins];   // per-wave digit counters, then exclusive wave bases
    __shared__ uint32_t s_dstart[kMaxBins];         // first LDS position of each digit in this tile
    __shared__ uint32_t s_goff[kMaxBins];           // global position of this tile's first pair of each digit
    __shared__ uint32_t s_scan[8];

    const int tid = threadIdx.x, lane = lane_id(), w = wave_id();
    const int bins = 1 << dbits;
    const uint32_t mask = (uint32_t)bins - 1u;
    const int64_t tile0 = (int64_t)blockIdx.x * kTile;
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
    {   // global base of every digit = scan of the digit totals, plus this tile's offset inside the digit
        uint32_t carry = 0;
        for (int base = 0; base < bins; base += kBlock) {
            const int d = base + tid;
            const uint32_t v = d < bins ? tot[d] : 0u;
            uint32_t total;
            const uint32_t ex = block_exclusive_scan(v, s_scan, &total);
            if (d < bins) s_goff[d] = carry + ex + hist[(int64_t)d * nb + blockIdx.x];
            carry += total;
        }
    }
    __syncthreads();

    // Stable rank of every pair among its wave's pairs of the same digit.  First the lanes of each round that share a
    // digit are matched (ballots only); then the first lane of each such set adds the set's size to the wave's counter
    // of the digit and gets back what was there -- the sets of a round have distinct digits, and a wave's LDS
    // operations are carried out in order, so the rounds' additions are issued back to back and need no barrier;
    // finally every lane takes that number from its set's first lane.
    uint32_t* wh = s_wh + w * kMaxBins;
    uint32_t old[ROUNDS];
    int lead[ROUNDS];
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) {
        const int p = w * kPerWave + r * kWave + lane;
        const bool valid = p < tile_n;
        const uint32_t d = (key[r] >> shift) & mask;
        const uint64_t m = match_digit(d, valid, dbits);
        const int rk = rank_below(m);
        lead[r] = valid ? __ffsll((unsigned long long)m) - 1 : lane;
        loc[r] = (uint32_t)rk;
        old[r] = 0u;
        if (valid && rk == 0) old[r] = atomicAdd(&wh[d], (uint32_t)__popcll(m));
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
            hipLaunchKernelGGL(k_sort_scan, dim3(1 << dbits), dim3(kBlock), 0, s, h->ws.sort_hist, nb, h->ws.sort_tot);
        }
        {
            Timed t(h, s, "sort_scatter");
            hipLaunchKernelGGL((k_sort_scatter<ROUNDS>), dim3(nb), dim3(kBlock), 0, s, key[*cur], val[*cur], key[*cur ^ 1],
                               val[*cur ^ 1], n, d_n, shift, dbits, h->ws.sort_hist, h->ws.sort_tot, nb);
        }
        *cur ^= 1;
    }
}

hipError_t launch_radix_sort_pairs(scars_handle* h, hipStream_t s, uint32_t* key[2], uint32_t* val[2], int64_t n,
                                   const int32_t* d_n, int bits, int* result_buffer) {
    int cur = 0;
    if (n > 0) {
        // small inputs: small tiles, so that there are enough workgroups to fill the chip
        if (n < ((int64_t)1 << 21)) sort_passes<kSortRoundsSmall>(h, s, key, val, n, d_n, bits, &cur);
        else sort_passes<kSortRoundsLarge>(h, s, key, val, n, d_n, bits, &cur);
    }
    *result_buffer = cur;
    return hipGetLastError();
}

}  // namespace scars
