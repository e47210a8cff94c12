// embedding_bag_bwd_update: sorted-segment scatter-add of the upstream gradient and the row update.
//
// Section IV of the paper splits an iteration into forward, backward and optimization and attributes the
// cost of the last two to writes of embedding rows (device memory for cached rows, host DRAM for the
// rest).  Here: (1) pairs (gid, bag) in position order; (2) stable radix sort by gid; (3) segment heads by
// ordered compaction (the integer outputs); (4) segment reduce in fixed chunks of kSegChunk sorted lookups
// per lane group -- a run that lies inside one chunk is summed and applied at once, a run that crosses
// chunk borders leaves one partial sum per chunk; (5) the chunk in which such a run starts adds the
// partials in chunk order and applies the update.  No floating-point atomics: results are bit-stable.
#include "scars_dev.h"

namespace scars {

// ---- (1) pairs ----------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void k_bwd_pairs(const int32_t* __restrict__ gid, const int32_t* __restrict__ off,
                                                      int64_t L, int64_t G, uint32_t* __restrict__ key,
                                                      uint32_t* __restrict__ val) {
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= L) return;
    // bag of position i: largest g with off[g] <= i  (empty bags share a start; the last of them owns nothing,
    // so step to the last g whose start is <= i)
    int64_t lo = 0, hi = G;   // answer in [lo, hi)
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if ((int64_t)off[mid] <= i) lo = mid; else hi = mid;
    }
    key[i] = (uint32_t)gid[i];   // -1 (invalid lookup) becomes the largest key and sorts last
    val[i] = (uint32_t)lo;
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
    uint32_t ca = 0, cb = 0;
    for (int base = 0; base < n; base += kBlock) {
        const int i = base + threadIdx.x;
        uint32_t va = i < n ? a[i] : 0u, vb = i < n ? b[i] : 0u, ta, tb;
        const uint32_t ea = block_exclusive_scan(va, s_scan, &ta);
        const uint32_t eb = block_exclusive_scan(vb, s_scan, &tb);
        if (i < n) { a[i] = ca + ea; b[i] = cb + eb; }
        ca += ta; cb += tb;
    }
    if (threadIdx.x == 0) { n_unique[0] = (int32_t)ca; n_unique[1] = (int32_t)cb; }
}

__global__ __launch_bounds__(kBlock) void k_seg_write(const uint32_t* __restrict__ key, const uint32_t* __restrict__ val,
                                                      int64_t L, const uint32_t* __restrict__ blk_head,
                                                      const int32_t* __restrict__ n_unique, int32_t* __restrict__ seg_start,
                                                      int32_t* __restrict__ unique_gid, int32_t* __restrict__ sorted_gid,
                                                      int32_t* __restrict__ sorted_bag) {
    __shared__ uint32_t s_a[4];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + wave_id() * kPerWaveS;
    bool hd[kRoundsS];
    uint32_t nh = 0;
#pragma unroll
    for (int r = 0; r < kRoundsS; ++r) {
        hd[r] = is_head(key, base + r * kWave + lane_id(), L);
        nh += (uint32_t)__popcll(ballot64(hd[r]));
    }
    if (lane_id() == 0) s_a[wave_id()] = nh;
    __syncthreads();
    uint32_t before = blk_head[blockIdx.x];
    for (int w = 0; w < wave_id(); ++w) before += s_a[w];
#pragma unroll
    for (int r = 0; r < kRoundsS; ++r) {
        const int64_t j = base + r * kWave + lane_id();
        const uint64_t m = ballot64(hd[r]);
        if (hd[r]) {
            const uint32_t u = before + (uint32_t)rank_below(m);
            seg_start[u] = (int32_t)j;
            unique_gid[u] = (int32_t)key[j];
        }
        before += (uint32_t)__popcll(m);
        if (sorted_gid && j < L) {   // caller asked for the sorted pairs as well
            sorted_gid[j] = (int32_t)key[j];
            sorted_bag[j] = (int32_t)val[j];
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) seg_start[n_unique[0]] = n_unique[1];
}

// ---- (4)/(5) segment reduce and update --------------------------------------------------------------------
struct UpdateArgs {
    const Meta* meta;
    const int32_t* slot_of;
    void* cache;
    float* state_cache;
    float lr, eps;
    int D;
};

// lane owns 4 consecutive columns [4*c, 4*c+4) of the row of `gid`; applies one optimizer step with gradient g.
// The step is evaluated in fp64 and rounded once: Adagrad from a zero accumulator is w -= lr*g/(|g|+eps), whose
// slope in g reaches lr/eps, so a gradient sum that is only fp32-accurate would miss a 1e-6 absolute bar.
template <int DTYPE, int OPT>
__device__ __forceinline__ void apply_update(const UpdateArgs& A, const int32_t* s_rbase, int T, int32_t gid, int c,
                                             const double (&g)[4]) {
    const int32_t slot = A.slot_of[gid];
    void* wrow;
    float* srow = nullptr;
    if (slot >= 0) {
        wrow = (char*)A.cache + (int64_t)slot * A.D * (DTYPE == SCARS_DTYPE_F32 ? 4 : 2);
        if (OPT == SCARS_OPT_ADAGRAD) srow = A.state_cache + (int64_t)slot * A.D;
    } else {
        const int t = upper_table(s_rbase, T, gid);
        const int64_t row = gid - s_rbase[t];
        wrow = (char*)A.meta->table[t] + row * A.D * (DTYPE == SCARS_DTYPE_F32 ? 4 : 2);
        if (OPT == SCARS_OPT_ADAGRAD) srow = A.meta->state[t] + row * A.D;
    }
    double w[4];
    if (DTYPE == SCARS_DTYPE_F32) {
        const float4 v = ((const float4*)wrow)[c];
        w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
    } else {
        const uint2 v = ((const uint2*)wrow)[c];
        w[0] = __uint_as_float(v.x << 16); w[1] = __uint_as_float(v.x & 0xFFFF0000u);
        w[2] = __uint_as_float(v.y << 16); w[3] = __uint_as_float(v.y & 0xFFFF0000u);
    }
    const double lr = (double)A.lr, eps = (double)A.eps;
    if (OPT == SCARS_OPT_SGD) {
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = w[i] - lr * g[i];
    } else {
        const float4 sv = ((const float4*)srow)[c];
        double st[4] = {sv.x, sv.y, sv.z, sv.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            st[i] = st[i] + g[i] * g[i];
            w[i] = w[i] - lr * g[i] / (sqrt(st[i]) + eps);
        }
        ((float4*)srow)[c] = make_float4((float)st[0], (float)st[1], (float)st[2], (float)st[3]);
    }
    if (DTYPE == SCARS_DTYPE_F32) {
        ((float4*)wrow)[c] = make_float4((float)w[0], (float)w[1], (float)w[2], (float)w[3]);
    } else {
        uint2 o;
        o.x = (uint32_t)f32_to_bf16((float)w[0]) | ((uint32_t)f32_to_bf16((float)w[1]) << 16);
        o.y = (uint32_t)f32_to_bf16((float)w[2]) | ((uint32_t)f32_to_bf16((float)w[3]) << 16);
        ((uint2*)wrow)[c] = o;
    }
}

// Group of LPG lanes per chunk of kSegChunk sorted lookups; lane c owns columns [4c, 4c+4).
// partial[(chunk*2 + side)*D + col]: side 0 = run open to the left (continues a previous chunk),
// side 1 = run that starts in this chunk and continues into the next.
template <int DTYPE, int OPT, int LPG>
__global__ __launch_bounds__(kBlock) void k_seg_reduce(const uint32_t* __restrict__ key, const uint32_t* __restrict__ val,
                                                       const int32_t* __restrict__ n_unique, const float* __restrict__ grad,
                                                       double* __restrict__ partial, UpdateArgs A) {
    __shared__ int32_t s_rbase[SCARS_MAX_TABLES + 1];
    const int T = A.meta->num_tables;
    for (int t = threadIdx.x; t <= T; t += kBlock) s_rbase[t] = A.meta->row_base[t];
    __syncthreads();
    const int64_t Lv = n_unique[1];
    const int64_t chunk = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / LPG;
    const int c = threadIdx.x % LPG;
    const int64_t j0 = chunk * kSegChunk;
    if (j0 >= Lv) return;
    const bool lane_on = c * 4 < A.D;
    const int64_t j1 = min(j0 + kSegChunk, Lv);
    const uint32_t none = 0xFFFFFFFFu;
    const uint32_t prev = j0 > 0 ? key[j0 - 1] : none;
    const uint32_t next = j1 < Lv ? key[j1] : none;
    uint32_t cur = key[j0];
    bool left_open = cur == prev;
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    const float4* g4 = (const float4*)grad;
    const int dq = A.D / 4;
    for (int64_t j = j0; j < j1; j += 4) {
        uint32_t kk[4];
        float4 gv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            kk[u] = none;
            if (j + u < j1) {
                kk[u] = key[j + u];
                if (lane_on) gv[u] = g4[(int64_t)val[j + u] * dq + c];
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (j + u < j1) {
                if (kk[u] != cur) {
                    // the run of `cur` ends inside this chunk
                    if (lane_on) {
                        if (left_open) {
                            double* p = partial + (chunk * 2 + 0) * A.D + c * 4;
                            p[0] = acc[0]; p[1] = acc[1]; p[2] = acc[2]; p[3] = acc[3];
                        } else {
                            apply_update<DTYPE, OPT>(A, s_rbase, T, (int32_t)cur, c, acc);
                        }
                    }
                    acc[0] = acc[1] = acc[2] = acc[3] = 0.0;
                    cur = kk[u];
                    left_open = false;
                }
                if (lane_on) { acc[0] += gv[u].x; acc[1] += gv[u].y; acc[2] += gv[u].z; acc[3] += gv[u].w; }
            }
        }
    }
    if (lane_on) {
        const bool right_open = cur == next;
        if (left_open) {
            double* p = partial + (chunk * 2 + 0) * A.D + c * 4;
            p[0] = acc[0]; p[1] = acc[1]; p[2] = acc[2]; p[3] = acc[3];
        } else if (right_open) {
            double* p = partial + (chunk * 2 + 1) * A.D + c * 4;
            p[0] = acc[0]; p[1] = acc[1]; p[2] = acc[2]; p[3] = acc[3];
        } else {
            apply_update<DTYPE, OPT>(A, s_rbase, T, (int32_t)cur, c, acc);
        }
    }
}

// The chunk in which a border-crossing run starts collects that run's partial sums in chunk order.
template <int DTYPE, int OPT, int LPG>
__global__ __launch_bounds__(kBlock) void k_seg_fixup(const uint32_t* __restrict__ key, const int32_t* __restrict__ n_unique,
                                                      const double* __restrict__ partial, UpdateArgs A) {
    __shared__ int32_t s_rbase[SCARS_MAX_TABLES + 1];
    const int T = A.meta->num_tables;
    for (int t = threadIdx.x; t <= T; t += kBlock) s_rbase[t] = A.meta->row_base[t];
    __syncthreads();
    const int64_t Lv = n_unique[1];
    const int64_t chunk = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / LPG;
    const int c = threadIdx.x % LPG;
    const int64_t j0 = chunk * kSegChunk;
    const int64_t j1 = j0 + kSegChunk;
    if (j1 >= Lv) return;                       // last chunk (or beyond): nothing continues to the right
    const uint32_t k = key[j1 - 1];
    if (key[j1] != k) return;                   // last run of this chunk ends at the border
    if (key[j0] == k && j0 > 0 && key[j0 - 1] == k) return;   // run started earlier: its first chunk collects
    if (c * 4 >= A.D) return;
    const double4* p4 = (const double4*)partial;
    const int dq = A.D / 4;
    double acc[4];
    {
        const double4 v = p4[(chunk * 2 + 1) * dq + c];
        acc[0] = v.x; acc[1] = v.y; acc[2] = v.z; acc[3] = v.w;
    }
    int64_t d = chunk + 1;
    while (d * kSegChunk < Lv && key[d * kSegChunk] == k) {
        double4 v[4];
        int n = 0;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if ((d + u) * kSegChunk < Lv && key[(d + u) * kSegChunk] == k) {
                v[u] = p4[((d + u) * 2 + 0) * dq + c];
                n = u + 1;
            } else {
                break;
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (u < n) { acc[0] += v[u].x; acc[1] += v[u].y; acc[2] += v[u].z; acc[3] += v[u].w; }
        d += n;
    }
    apply_update<DTYPE, OPT>(A, s_rbase, T, (int32_t)k, c, acc);
}

template <int DTYPE, int OPT, int LPG>
static void launch_reduce_t(scars_handle* h, hipStream_t s, const uint32_t* key, const uint32_t* val, const int32_t* nu,
                            const float* grad, int64_t L, UpdateArgs A) {
    const int64_t chunks = div_up(L, kSegChunk);
    const unsigned grid = (unsigned)div_up(chunks * LPG, kBlock);
    {
        Timed t(h, s, "seg_reduce");
        hipLaunchKernelGGL((k_seg_reduce<DTYPE, OPT, LPG>), dim3(grid), dim3(kBlock), 0, s, key, val, nu, grad,
                           h->ws.partial, A);
    }
    {
        Timed t(h, s, "seg_fixup");
        hipLaunchKernelGGL((k_seg_fixup<DTYPE, OPT, LPG>), dim3(grid), dim3(kBlock), 0, s, key, nu, h->ws.partial, A);
    }
}

template <int DTYPE, int OPT>
static void launch_reduce_o(int lpg, scars_handle* h, hipStream_t s, const uint32_t* key, const uint32_t* val,
                            const int32_t* nu, const float* grad, int64_t L, UpdateArgs A) {
    switch (lpg) {
#define SCARS_CASE(N) case N: launch_reduce_t<DTYPE, OPT, N>(h, s, key, val, nu, grad, L, A); break;
        SCARS_CASE(1) SCARS_CASE(2) SCARS_CASE(4) SCARS_CASE(8) SCARS_CASE(16) SCARS_CASE(32) SCARS_CASE(64)
        SCARS_CASE(128)
#undef SCARS_CASE
    }
}

hipError_t launch_bwd(scars_handle* h, hipStream_t s, const int32_t* off, int64_t L, int64_t B,
                      const scars_remap_out* rm, const float* grad, float lr, float eps, const scars_bwd_out* out) {
    Workspace& ws = h->ws;
    int32_t* n_unique = out ? out->n_unique : ws.n_unique;
    int32_t* seg_start = out ? out->seg_start : ws.seg_start;
    int32_t* unique_gid = out ? out->unique_gid : ws.unique_gid;
    const int64_t G = (int64_t)h->T * B;
    if (L == 0) {
        Timed t(h, s, "bwd_empty");
        hipLaunchKernelGGL(k_bwd_empty, dim3(1), dim3(kWave), 0, s, n_unique, seg_start);
        return hipGetLastError();
    }
    {
        Timed t(h, s, "bwd_pairs");
        hipLaunchKernelGGL(k_bwd_pairs, dim3((unsigned)div_up(L, kBlock)), dim3(kBlock), 0, s, rm->gid, off, L, G,
                           ws.key_buf[0], ws.val_buf[0]);
    }
    int bits = 1;
    while (bits < 32 && ((int64_t)1 << bits) <= h->N) ++bits;   // 2^bits - 1 >= N: the sentinel stays the largest key
    int res = 0;
    hipError_t e = launch_radix_sort_pairs(h, s, ws.key_buf, ws.val_buf, L, bits, &res);
    if (e != hipSuccess) return e;
    const uint32_t* key = ws.key_buf[res];
    const uint32_t* val = ws.val_buf[res];
    const int nb = (int)div_up(L, kScanTile);
    {
        Timed t(h, s, "seg_count");
        hipLaunchKernelGGL(k_seg_count, dim3(nb), dim3(kBlock), 0, s, key, L, ws.blk_hit, ws.blk_miss);
    }
    {
        Timed t(h, s, "seg_scan");
        hipLaunchKernelGGL(k_seg_scan, dim3(1), dim3(kBlock), 0, s, ws.blk_hit, ws.blk_miss, nb, n_unique);
    }
    {
        Timed t(h, s, "seg_write");
        hipLaunchKernelGGL(k_seg_write, dim3(nb), dim3(kBlock), 0, s, key, val, L, ws.blk_hit, n_unique, seg_start,
                           unique_gid, out ? out->sorted_gid : nullptr, out ? out->sorted_bag : nullptr);
    }
    UpdateArgs A{ws.meta, h->buf.slot_of, h->buf.cache, h->buf.state_cache, lr, eps, h->D};
    const int lpg = next_pow2_host(h->D / 4);
    if (h->dtype == SCARS_DTYPE_F32) {
        if (h->optimizer == SCARS_OPT_SGD) launch_reduce_o<SCARS_DTYPE_F32, SCARS_OPT_SGD>(lpg, h, s, key, val, n_unique, grad, L, A);
        else launch_reduce_o<SCARS_DTYPE_F32, SCARS_OPT_ADAGRAD>(lpg, h, s, key, val, n_unique, grad, L, A);
    } else {
        if (h->optimizer == SCARS_OPT_SGD) launch_reduce_o<SCARS_DTYPE_BF16, SCARS_OPT_SGD>(lpg, h, s, key, val, n_unique, grad, L, A);
        else launch_reduce_o<SCARS_DTYPE_BF16, SCARS_OPT_ADAGRAD>(lpg, h, s, key, val, n_unique, grad, L, A);
    }
    return hipGetLastError();
}

}  // namespace scars
