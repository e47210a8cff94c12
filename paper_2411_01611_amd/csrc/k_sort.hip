// Stable LSD radix sort of (uint32 key, uint32 value) pairs, 8 bits per pass, staged through LDS.
//
// Used for (a) ordering the selected hot rows by descending count (key = ~count, value = gid; the input is
// in ascending gid order, so stability gives "lower id first among equal counts"), and (b) ordering a
// batch's lookups by (gid, position) for the backward pass (key = gid, value = bag; the input is in
// position order).  Per pass: per-tile digit histogram -> per-digit exclusive scan over tiles -> scatter
// in which each tile is first ordered in LDS (wave-level multi-split by ballot matching) and then written
// out as contiguous runs per digit.
#include "scars_dev.h"

namespace scars {

constexpr int kItemsPerWave = kSortTile / (kBlock / kWave);   // 1024
constexpr int kRounds = kItemsPerWave / kWave;                // 16

__global__ __launch_bounds__(kBlock) void k_sort_hist(const uint32_t* __restrict__ keys, int64_t n, int shift,
                                                      uint32_t* __restrict__ hist, int nb) {
    __shared__ uint32_t s_hist[256];
    s_hist[threadIdx.x] = 0;
    __syncthreads();
    const int64_t tile0 = (int64_t)blockIdx.x * kSortTile;
#pragma unroll 4
    for (int r = 0; r < kSortTile / kBlock; ++r) {
        int64_t i = tile0 + (int64_t)r * kBlock + threadIdx.x;
        if (i < n) atomicAdd(&s_hist[(keys[i] >> shift) & 0xFFu], 1u);
    }
    __syncthreads();
    hist[(int64_t)threadIdx.x * nb + blockIdx.x] = s_hist[threadIdx.x];
}

// One workgroup per digit: exclusive scan of that digit's per-tile counts, digit total to tot[digit].
__global__ __launch_bounds__(kBlock) void k_sort_scan(uint32_t* __restrict__ hist, int nb, uint32_t* __restrict__ tot) {
    __shared__ uint32_t s_scan[8];
    uint32_t* row = hist + (int64_t)blockIdx.x * nb;
    uint32_t carry = 0;
    for (int base = 0; base < nb; base += kBlock) {
        int i = base + threadIdx.x;
        uint32_t v = i < nb ? row[i] : 0u;
        uint32_t total;
        uint32_t ex = block_exclusive_scan(v, s_scan, &total);
        if (i < nb) row[i] = carry + ex;
        carry += total;
    }
    if (threadIdx.x == 0) tot[blockIdx.x] = carry;
}

__global__ __launch_bounds__(kBlock) void k_sort_scatter(const uint32_t* __restrict__ kin, const uint32_t* __restrict__ vin,
                                                         uint32_t* __restrict__ kout, uint32_t* __restrict__ vout,
                                                         int64_t n, int shift, const uint32_t* __restrict__ hist,
                                                         const uint32_t* __restrict__ tot, int nb) {
    __shared__ uint32_t s_key[kSortTile];
    __shared__ uint32_t s_val[kSortTile];
    __shared__ uint32_t s_wh[(kBlock / kWave) * 256];   // per-wave digit counters, then wave bases
    __shared__ uint32_t s_dstart[256];                   // first LDS position of each digit in this tile
    __shared__ uint32_t s_goff[256];                     // global position of this tile's first item of each digit
    __shared__ uint32_t s_scan[8];

    const int tid = threadIdx.x, lane = lane_id(), w = wave_id();
    const int64_t tile0 = (int64_t)blockIdx.x * kSortTile;
    const int tile_n = (int)min((int64_t)kSortTile, n - tile0);

    for (int i = tid; i < (kBlock / kWave) * 256; i += kBlock) s_wh[i] = 0;
    {   // global base of every digit = scan of the digit totals, plus this tile's offset inside the digit
        uint32_t total;
        uint32_t ex = block_exclusive_scan(tot[tid], s_scan, &total);
        s_goff[tid] = ex + hist[(int64_t)tid * nb + blockIdx.x];
    }
    __syncthreads();

    uint32_t key[kRounds], val[kRounds], loc[kRounds];
    volatile uint32_t* wh = s_wh + w * 256;
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int p = w * kItemsPerWave + r * kWave + lane;     // position inside the tile
        const bool valid = p < tile_n;
        key[r] = valid ? kin[tile0 + p] : 0xFFFFFFFFu;
        val[r] = valid ? vin[tile0 + p] : 0u;
        const uint32_t d = (key[r] >> shift) & 0xFFu;
        // lanes holding the same digit
        uint64_t m = ballot64(valid);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const bool bit = (d >> b) & 1u;
            const uint64_t bal = ballot64(bit);
            m &= bit ? bal : ~bal;
        }
        const uint32_t before = valid ? wh[d] : 0u;
        __builtin_amdgcn_wave_barrier();
        const int rk = rank_below(m);
        if (valid && rk == 0) wh[d] = before + (uint32_t)__popcll(m);
        __builtin_amdgcn_wave_barrier();
        loc[r] = before + (uint32_t)rk;                          // stable rank among this wave's items of digit d
    }
    __syncthreads();
    {   // per digit: wave counts -> exclusive wave bases; tile count of the digit -> LDS start of the digit
        uint32_t run = 0;
#pragma unroll
        for (int ww = 0; ww < kBlock / kWave; ++ww) {
            uint32_t t = s_wh[ww * 256 + tid];
            s_wh[ww * 256 + tid] = run;
            run += t;
        }
        uint32_t total;
        s_dstart[tid] = block_exclusive_scan(run, s_scan, &total);
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int p = w * kItemsPerWave + r * kWave + lane;
        if (p < tile_n) {
            const uint32_t d = (key[r] >> shift) & 0xFFu;
            const uint32_t q = s_dstart[d] + s_wh[w * 256 + d] + loc[r];
            s_key[q] = key[r];
            s_val[q] = val[r];
        }
    }
    __syncthreads();
    for (int q = tid; q < tile_n; q += kBlock) {
        const uint32_t k = s_key[q];
        const uint32_t d = (k >> shift) & 0xFFu;
        const uint32_t dst = s_goff[d] + ((uint32_t)q - s_dstart[d]);
        kout[dst] = k;
        vout[dst] = s_val[q];
    }
}

hipError_t launch_radix_sort_pairs(scars_handle* h, hipStream_t s, uint32_t* key[2], uint32_t* val[2], int64_t n,
                                   int bits, int* result_buffer) {
    int cur = 0;
    if (n > 0) {
        const int nb = (int)div_up(n, kSortTile);
        for (int shift = 0; shift < bits; shift += 8) {
            {
                Timed t(h, s, "sort_hist");
                hipLaunchKernelGGL(k_sort_hist, dim3(nb), dim3(kBlock), 0, s, key[cur], n, shift, h->ws.sort_hist, nb);
            }
            {
                Timed t(h, s, "sort_scan");
                hipLaunchKernelGGL(k_sort_scan, dim3(256), dim3(kBlock), 0, s, h->ws.sort_hist, nb, h->ws.sort_tot);
            }
            {
                Timed t(h, s, "sort_scatter");
                hipLaunchKernelGGL(k_sort_scatter, dim3(nb), dim3(kBlock), 0, s, key[cur], val[cur], key[cur ^ 1],
                                   val[cur ^ 1], n, shift, h->ws.sort_hist, h->ws.sort_tot, nb);
            }
            cur ^= 1;
        }
    }
    *result_buffer = cur;
    return hipGetLastError();
}

}  // namespace scars
