// classify_samples: hot / normal samples of a batch and their stable partition.
//
// Section III of the paper sorts training samples into "hot" ones, which need only cached embeddings, and
// "normal" ones, and composes mini-batches of one kind.  A sample is hot when none of its lookups, over all
// tables, is a miss (a sample without lookups is hot).  One thread per sample reads the slots written by
// remap; the sample ids of each class are then listed in ascending order by the same tile-count / scan /
// write compaction as the hit and miss lists.
#include "scars_dev.h"

namespace scars {

constexpr int kPerWaveC = kScanTile / (kBlock / kWave);   // 512 consecutive samples per wave
constexpr int kRoundsC = kPerWaveC / kWave;               // 8 rounds of 64

__global__ __launch_bounds__(kBlock) void k_cls_flag(const int32_t* __restrict__ off, int32_t L, int64_t B, int T,
                                                     const int32_t* __restrict__ slot, const int32_t* __restrict__ gid,
                                                     int32_t* __restrict__ is_hot, uint32_t* __restrict__ blk_hot,
                                                     uint32_t* __restrict__ blk_normal) {
    __shared__ uint32_t s_h[4], s_n[4];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + wave_id() * kPerWaveC;
    uint32_t nh = 0, nn = 0;
#pragma unroll 1
    for (int r = 0; r < kRoundsC; ++r) {
        const int64_t b = base + r * kWave + lane_id();
        bool hot = true;
        if (b < B) {
            for (int t = 0; t < T; ++t) {
                const int64_t g = (int64_t)t * B + b;
                const int32_t a = min(max(off[g], 0), L);
                const int32_t e = min(max(off[g + 1], a), L);
                for (int32_t i = a; i < e; ++i)
                    if (gid[i] >= 0 && slot[i] < 0) hot = false;
            }
            is_hot[b] = hot ? 1 : 0;
        }
        nh += (uint32_t)__popcll(ballot64(b < B && hot));
        nn += (uint32_t)__popcll(ballot64(b < B && !hot));
    }
    if (lane_id() == 0) { s_h[wave_id()] = nh; s_n[wave_id()] = nn; }
    __syncthreads();
    if (threadIdx.x == 0) {
        blk_hot[blockIdx.x] = s_h[0] + s_h[1] + s_h[2] + s_h[3];
        blk_normal[blockIdx.x] = s_n[0] + s_n[1] + s_n[2] + s_n[3];
    }
}

__global__ __launch_bounds__(kBlock) void k_cls_write(const int32_t* __restrict__ is_hot, int64_t B,
                                                      const uint32_t* __restrict__ blk_hot, const uint32_t* __restrict__ blk_normal,
                                                      int scanned, int32_t* __restrict__ n_hot_normal,
                                                      int32_t* __restrict__ hot_ids, int32_t* __restrict__ normal_ids) {
    __shared__ uint32_t s_h[4], s_n[4], s_red[8];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + wave_id() * kPerWaveC;
    int32_t f[kRoundsC];
    uint32_t nh = 0, nn = 0;
#pragma unroll
    for (int r = 0; r < kRoundsC; ++r) {
        const int64_t b = base + r * kWave + lane_id();
        f[r] = b < B ? is_hot[b] : -1;
        nh += (uint32_t)__popcll(ballot64(f[r] == 1));
        nn += (uint32_t)__popcll(ballot64(f[r] == 0));
    }
    if (lane_id() == 0) { s_h[wave_id()] = nh; s_n[wave_id()] = nn; }
    __syncthreads();
    uint32_t hb, nb, th, tn;
    tile_prefix2(blk_hot, blk_normal, blockIdx.x, gridDim.x, scanned != 0, s_red, n_hot_normal, &hb, &nb, &th, &tn);
    for (int w = 0; w < wave_id(); ++w) { hb += s_h[w]; nb += s_n[w]; }
#pragma unroll
    for (int r = 0; r < kRoundsC; ++r) {
        const int64_t b = base + r * kWave + lane_id();
        const uint64_t mh = ballot64(f[r] == 1), mn = ballot64(f[r] == 0);
        if (f[r] == 1) hot_ids[hb + rank_below(mh)] = (int32_t)b;
        else if (f[r] == 0) normal_ids[nb + rank_below(mn)] = (int32_t)b;
        hb += (uint32_t)__popcll(mh);
        nb += (uint32_t)__popcll(mn);
    }
}

// Use of the cache by portion (the measurement behind Fig. 4 of the paper): usage[p] = samples with at least one
// lookup whose slot lies in [p * portion_rows, (p + 1) * portion_rows).  One thread per sample builds a bit mask
// of the portions it touches; one integer atomic per wave and portion.
__global__ __launch_bounds__(kBlock) void k_portion_usage(const int32_t* __restrict__ off, int32_t L, int64_t B, int T,
                                                          const int32_t* __restrict__ slot, int32_t portion_rows,
                                                          int n_portions, int32_t* __restrict__ usage) {
    const int64_t b = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    uint64_t mask = 0;
    if (b < B) {
        for (int t = 0; t < T; ++t) {
            const int64_t g = (int64_t)t * B + b;
            const int32_t a = min(max(off[g], 0), L);
            const int32_t e = min(max(off[g + 1], a), L);
            for (int32_t i = a; i < e; ++i) {
                const int32_t s = slot[i];
                if (s >= 0 && s / portion_rows < n_portions) mask |= 1ull << (s / portion_rows);
            }
        }
    }
    for (int p = 0; p < n_portions; ++p) {
        const int c = __popcll(ballot64((mask >> p) & 1ull));
        if (c && lane_id() == 0) atomicAdd(&usage[p], c);
    }
}

hipError_t launch_portion_usage(scars_handle* h, hipStream_t s, const int32_t* off, int64_t L, int64_t B,
                                const scars_remap_out* rm, int64_t portion_rows, int32_t n_portions, int32_t* usage) {
    hipError_t e = launch_fill_u32(h, s, (uint32_t*)usage, n_portions, 0u);
    if (e != hipSuccess) return e;
    if (B > 0) {
        Timed t(h, s, "portion_usage");
        hipLaunchKernelGGL(k_portion_usage, dim3((unsigned)div_up(B, kBlock)), dim3(kBlock), 0, s, off, (int32_t)L, B, h->T,
                           rm->slot, (int32_t)std::min<int64_t>(portion_rows, 0x7fffffff), n_portions, usage);
    }
    return hipGetLastError();
}

// ---- sub-batch of selected samples (Section III: hot and normal samples go to separate mini-batches) ---------
// Bag t*n + j of the sub-batch is bag t*B + ids[j] of the batch.  Same count / (scan) / write scheme as the other
// compactions, with bag lengths in place of flags: a tile is 2048 bags of the sub-batch.
__device__ __forceinline__ int32_t sub_bag(const int32_t* __restrict__ off, const int32_t* __restrict__ ids, int64_t gs,
                                           int64_t n, int64_t B, int32_t L, int32_t* a_out) {
    // gs < T*n.  Returns the bag's length, its first lookup in *a_out (offsets and ids clamped into range)
    const int64_t t = gs / n, j = gs - t * n;
    const int64_t b = min(max((int64_t)ids[j], (int64_t)0), B - 1);
    const int64_t g = t * B + b;
    const int32_t a = min(max(off[g], 0), L);
    const int32_t e = min(max(off[g + 1], a), L);
    *a_out = a;
    return e - a;
}

__global__ __launch_bounds__(kBlock) void k_part_count(const int32_t* __restrict__ off, const int32_t* __restrict__ ids,
                                                       const int32_t* __restrict__ d_n, int64_t B, int T, int32_t L,
                                                       uint32_t* __restrict__ blk_len, uint32_t* __restrict__ blk_bags) {
    __shared__ uint32_t s_a[4], s_b[4];
    const int64_t n = min(max((int64_t)*d_n, (int64_t)0), B);
    const int64_t Gs = (int64_t)T * n;
    const int64_t base = (int64_t)blockIdx.x * kScanTile + wave_id() * kPerWaveC;
    uint32_t sum = 0, bags = 0;
#pragma unroll 1
    for (int r = 0; r < kRoundsC; ++r) {
        const int64_t gs = base + r * kWave + lane_id();
        int32_t a;
        const uint32_t len = gs < Gs ? (uint32_t)sub_bag(off, ids, gs, n, B, L, &a) : 0u;
        sum += wave_sum(len);
        bags += (uint32_t)__popcll(ballot64(gs < Gs));
    }
    if (lane_id() == 0) { s_a[wave_id()] = sum; s_b[wave_id()] = bags; }
    __syncthreads();
    if (threadIdx.x == 0) {
        blk_len[blockIdx.x] = s_a[0] + s_a[1] + s_a[2] + s_a[3];
        blk_bags[blockIdx.x] = s_b[0] + s_b[1] + s_b[2] + s_b[3];
    }
}

__global__ __launch_bounds__(kBlock) void k_part_write(const int32_t* __restrict__ idx, const int32_t* __restrict__ off,
                                                       const int32_t* __restrict__ ids, const int32_t* __restrict__ d_n,
                                                       int64_t B, int T, int32_t L, const uint32_t* __restrict__ blk_len,
                                                       const uint32_t* __restrict__ blk_bags, int scanned,
                                                       int32_t* __restrict__ n_out, int32_t* __restrict__ sub_idx,
                                                       int32_t* __restrict__ sub_off) {
    __shared__ uint32_t s_w[4], s_red[8];
    const int64_t n = min(max((int64_t)*d_n, (int64_t)0), B);
    const int64_t Gs = (int64_t)T * n;
    const int64_t base = (int64_t)blockIdx.x * kScanTile + wave_id() * kPerWaveC;
    // lengths of this wave's 512 bags, 8 rounds of 64
    uint32_t len[kRoundsC];
    int32_t first[kRoundsC];
    uint32_t wsum = 0;
#pragma unroll
    for (int r = 0; r < kRoundsC; ++r) {
        const int64_t gs = base + r * kWave + lane_id();
        first[r] = 0;
        len[r] = gs < Gs ? (uint32_t)sub_bag(off, ids, gs, n, B, L, &first[r]) : 0u;
        wsum += wave_sum(len[r]);
    }
    if (lane_id() == 0) s_w[wave_id()] = wsum;
    __syncthreads();
    uint32_t before, bags_before, tl, tb;
    tile_prefix2(blk_len, blk_bags, blockIdx.x, gridDim.x, scanned != 0, s_red, n_out, &before, &bags_before, &tl, &tb);
    for (int w = 0; w < wave_id(); ++w) before += s_w[w];
    if (blockIdx.x == 0 && threadIdx.x == 0) sub_off[0] = 0;
#pragma unroll
    for (int r = 0; r < kRoundsC; ++r) {
        const int64_t gs = base + r * kWave + lane_id();
        const uint32_t inc = wave_inclusive_scan(len[r]);
        if (gs < Gs) {
            const uint32_t start = before + inc - len[r];
            sub_off[gs + 1] = (int32_t)(before + inc);
            // (after an offsets error bags may overlap and their lengths add up to more than L: never write past L)
            for (uint32_t i = 0; i < len[r] && start + i < (uint32_t)L; ++i) sub_idx[start + i] = idx[first[r] + (int32_t)i];
        }
        before += __shfl(inc, kWave - 1, kWave);
    }
}

hipError_t launch_partition(scars_handle* h, hipStream_t s, const int32_t* idx, const int32_t* off, int64_t L, int64_t B,
                            const int32_t* ids, const int32_t* d_n, const scars_subbatch_out* out) {
    Workspace& ws = h->ws;
    const int nb = (int)std::max<int64_t>(1, div_up((int64_t)h->T * B, kScanTile));
    {
        Timed t(h, s, "part_count");
        hipLaunchKernelGGL(k_part_count, dim3(nb), dim3(kBlock), 0, s, off, ids, d_n, B, h->T, (int32_t)L, ws.blk_hit,
                           ws.blk_miss);
    }
    const bool scan = nb > h->fused_scan_max_tiles;
    if (scan) {
        Timed t(h, s, "part_scan");
        hipLaunchKernelGGL(k_remap_scan, dim3(1), dim3(kBlock), 0, s, ws.blk_hit, ws.blk_miss, nb, out->n_lookups_bags);
    }
    {
        Timed t(h, s, "part_write");
        hipLaunchKernelGGL(k_part_write, dim3(nb), dim3(kBlock), 0, s, idx, off, ids, d_n, B, h->T, (int32_t)L, ws.blk_hit,
                           ws.blk_miss, scan ? 1 : 0, out->n_lookups_bags, out->indices, out->offsets);
    }
    return hipGetLastError();
}

hipError_t launch_classify(scars_handle* h, hipStream_t s, const int32_t* off, int64_t L, int64_t B,
                           const scars_remap_out* rm, const scars_classify_out* out) {
    Workspace& ws = h->ws;
    const int nb = (int)std::max<int64_t>(1, div_up(B, kScanTile));
    {
        Timed t(h, s, "cls_flag");
        hipLaunchKernelGGL(k_cls_flag, dim3(nb), dim3(kBlock), 0, s, off, (int32_t)L, B, h->T, rm->slot, rm->gid,
                           out->is_hot, ws.blk_hit, ws.blk_miss);
    }
    const bool scan = nb > h->fused_scan_max_tiles;   // few tiles: the writer adds up the tile counts itself
    if (scan) {
        Timed t(h, s, "cls_scan");
        hipLaunchKernelGGL(k_remap_scan, dim3(1), dim3(kBlock), 0, s, ws.blk_hit, ws.blk_miss, nb, out->n_hot_normal);
    }
    {
        Timed t(h, s, "cls_write");
        hipLaunchKernelGGL(k_cls_write, dim3(nb), dim3(kBlock), 0, s, out->is_hot, B, ws.blk_hit, ws.blk_miss,
                           scan ? 1 : 0, out->n_hot_normal, out->hot_ids, out->normal_ids);
    }
    return hipGetLastError();
}

}  // namespace scars
