// remap: index -> cache slot, with ordered (stable) compaction of hit and miss positions.
//
// Section II-B caches a set C of embeddings on the device; Section IV observes that the lookup into that
// cached layer bounds the forward pass.  Here one pass maps every lookup to gid = row_base[t] + idx and
// slot = slot_of[gid] (a dense int32 map, one random 4-byte read), and a three-kernel ordered compaction
// (per-tile counts -> scan -> write) lists hits and misses in ascending position, so that the lists are
// unique and comparable bit for bit.  loc[i] tells the forward kernel where to read the row: the cache slot
// for a hit, k + rank-in-miss-list (a row of the staging area) for a miss.
#include <mutex>

#include "scars_dev.h"

namespace scars {

constexpr int kPerWave = kScanTile / (kBlock / kWave);   // 512 consecutive lookups per wave
constexpr int kRoundsR = kPerWave / kWave;               // 8 rounds of 64

__global__ __launch_bounds__(kBlock) void k_remap_probe(const int32_t* __restrict__ idx, const int32_t* __restrict__ off,
                                                        int64_t L, int64_t B, const Meta* __restrict__ meta,
                                                        const int32_t* __restrict__ slot_of, int32_t* __restrict__ slot,
                                                        int32_t* __restrict__ gid, uint32_t* __restrict__ blk_hit,
                                                        uint32_t* __restrict__ blk_miss, int32_t* __restrict__ status) {
    __shared__ int32_t s_tstart[SCARS_MAX_TABLES + 1];
    __shared__ int32_t s_rbase[SCARS_MAX_TABLES + 1];
    __shared__ uint32_t s_hit[4], s_miss[4];
    const int T = meta->num_tables;
    for (int t = threadIdx.x; t <= T; t += kBlock) {
        const int32_t v = off[(int64_t)t * B];
        s_tstart[t] = v;
        s_rbase[t] = meta->row_base[t];
    }
    __syncthreads();
    const int64_t G = (int64_t)T * B;
    const int64_t nthreads = (int64_t)gridDim.x * kBlock;
    const int64_t gt = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    for (int64_t g = gt; g < G; g += nthreads)
        if (off[g + 1] < off[g]) latch_error(status, SCARS_ERR_OFFSETS);
    if (gt == 0 && (off[0] != 0 || (int64_t)off[G] != L)) latch_error(status, SCARS_ERR_OFFSETS);

    const int64_t base = (int64_t)blockIdx.x * kScanTile + wave_id() * kPerWave;
    uint32_t nh = 0, nm = 0;
    // positions are clamped instead of guarded so that the index loads of all rounds, then the slot probes of
    // all rounds, are issued back to back; only positions below L are written and counted
    int32_t row[kRoundsR], g[kRoundsR], sl[kRoundsR];
    const int64_t last = L - 1;
    if (L > 0) {
#pragma unroll
        for (int r = 0; r < kRoundsR; ++r) row[r] = idx[min(base + r * kWave + lane_id(), last)];
#pragma unroll
        for (int r = 0; r < kRoundsR; ++r) {
            const int64_t i = min(base + r * kWave + lane_id(), last);
            const int t = upper_table(s_tstart, T, (int32_t)i);
            const int32_t nrows = s_rbase[t + 1] - s_rbase[t];
            g[r] = (row[r] < 0 || row[r] >= nrows) ? -1 : s_rbase[t] + row[r];
        }
#pragma unroll
        for (int r = 0; r < kRoundsR; ++r) sl[r] = slot_of[max(g[r], 0)];
    }
#pragma unroll
    for (int r = 0; r < kRoundsR; ++r) {
        const int64_t i = base + r * kWave + lane_id();
        bool hit = false, miss = false;
        if (i < L) {
            if (g[r] < 0) {
                latch_error(status, SCARS_ERR_INDEX_RANGE);
                sl[r] = -1;
            }
            hit = sl[r] >= 0;
            miss = g[r] >= 0 && !hit;
            slot[i] = sl[r];
            gid[i] = g[r];
        }
        nh += (uint32_t)__popcll(ballot64(hit));
        nm += (uint32_t)__popcll(ballot64(miss));
    }
    if (lane_id() == 0) { s_hit[wave_id()] = nh; s_miss[wave_id()] = nm; }
    __syncthreads();
    if (threadIdx.x == 0) {
        blk_hit[blockIdx.x] = s_hit[0] + s_hit[1] + s_hit[2] + s_hit[3];
        blk_miss[blockIdx.x] = s_miss[0] + s_miss[1] + s_miss[2] + s_miss[3];
    }
}

// single workgroup: exclusive scan of the per-tile counts; totals to n_hit_miss[2] (and a[n], b[n])
__global__ __launch_bounds__(kBlock) void k_remap_scan(uint32_t* __restrict__ a, uint32_t* __restrict__ b, int n,
                                                       int32_t* __restrict__ n_hit_miss) {
    __shared__ uint32_t s_scan[8];
    uint32_t ca, cb;
    scan_two_counts(a, b, n, s_scan, &ca, &cb);
    if (threadIdx.x == 0) {
        a[n] = ca; b[n] = cb;
        n_hit_miss[0] = (int32_t)ca;
        n_hit_miss[1] = (int32_t)cb;
    }
}

// tile `tile` of `ntiles`
__device__ __forceinline__ void remap_write_body(int tile, int ntiles, int64_t L, const int32_t* __restrict__ slot,
                                                 const int32_t* __restrict__ gid, const uint32_t* __restrict__ blk_hit,
                                                 const uint32_t* __restrict__ blk_miss, int scanned,
                                                 int32_t* __restrict__ n_hit_miss, int32_t k, int32_t* __restrict__ loc,
                                                 int32_t* __restrict__ hit_pos, int32_t* __restrict__ miss_pos,
                                                 int32_t* __restrict__ miss_gid) {
    __shared__ uint32_t s_hit[4], s_miss[4], s_red[8];
    const int64_t base = (int64_t)tile * kScanTile + wave_id() * kPerWave;
    int32_t s[kRoundsR], g[kRoundsR];
    uint32_t nh = 0, nm = 0;
#pragma unroll
    for (int r = 0; r < kRoundsR; ++r) {
        const int64_t i = base + r * kWave + lane_id();
        s[r] = i < L ? slot[i] : -1;
        g[r] = i < L ? gid[i] : -1;
        nh += (uint32_t)__popcll(ballot64(s[r] >= 0));
        nm += (uint32_t)__popcll(ballot64(s[r] < 0 && g[r] >= 0));
    }
    if (lane_id() == 0) { s_hit[wave_id()] = nh; s_miss[wave_id()] = nm; }
    __syncthreads();
    uint32_t hb, mb, th, tm;
    tile_prefix2(blk_hit, blk_miss, tile, ntiles, scanned != 0, s_red, n_hit_miss, &hb, &mb, &th, &tm);
    for (int w = 0; w < wave_id(); ++w) { hb += s_hit[w]; mb += s_miss[w]; }
#pragma unroll
    for (int r = 0; r < kRoundsR; ++r) {
        const int64_t i = base + r * kWave + lane_id();
        const bool hit = s[r] >= 0, miss = s[r] < 0 && g[r] >= 0;
        const uint64_t mh = ballot64(hit), mm = ballot64(miss);
        if (hit) {
            hit_pos[hb + rank_below(mh)] = (int32_t)i;
            loc[i] = s[r];
        } else if (miss) {
            const uint32_t j = mb + rank_below(mm);
            miss_pos[j] = (int32_t)i;
            miss_gid[j] = g[r];
            loc[i] = k + (int32_t)j;
        } else if (i < L) {
            loc[i] = -1;
        }
        hb += (uint32_t)__popcll(mh);
        mb += (uint32_t)__popcll(mm);
    }
}

__global__ __launch_bounds__(kBlock) void k_remap_write(int64_t L, const int32_t* __restrict__ slot,
                                                        const int32_t* __restrict__ gid, const uint32_t* __restrict__ blk_hit,
                                                        const uint32_t* __restrict__ blk_miss, int scanned,
                                                        int32_t* __restrict__ n_hit_miss, int32_t k,
                                                        int32_t* __restrict__ loc, int32_t* __restrict__ hit_pos,
                                                        int32_t* __restrict__ miss_pos, int32_t* __restrict__ miss_gid) {
    remap_write_body((int)blockIdx.x, (int)gridDim.x, L, slot, gid, blk_hit, blk_miss, scanned, n_hit_miss, k, loc, hit_pos,
                     miss_pos, miss_gid);
}

// The same, and in the other workgroups of the launch the (gid, bag) pairs the backward pass of this batch will sort:
// both read what k_remap_probe wrote and nothing of each other, so the pairs cost no launch of their own.
__global__ __launch_bounds__(kBlock) void k_remap_write_pairs(int ntiles, int64_t L, const int32_t* __restrict__ slot,
                                                              const int32_t* __restrict__ gid,
                                                              const uint32_t* __restrict__ blk_hit,
                                                              const uint32_t* __restrict__ blk_miss, int scanned,
                                                              int32_t* __restrict__ n_hit_miss, int32_t k,
                                                              int32_t* __restrict__ loc, int32_t* __restrict__ hit_pos,
                                                              int32_t* __restrict__ miss_pos, int32_t* __restrict__ miss_gid,
                                                              const int32_t* __restrict__ off, int64_t G, int lpb,
                                                              int shift, uint32_t* __restrict__ key,
                                                              uint32_t* __restrict__ val) {
    if ((int)blockIdx.x < ntiles)
        remap_write_body((int)blockIdx.x, ntiles, L, slot, gid, blk_hit, blk_miss, scanned, n_hit_miss, k, loc, hit_pos,
                         miss_pos, miss_gid);
    else
        bag_pairs((int64_t)blockIdx.x - ntiles, gid, off, (int32_t)L, G, lpb, shift, key, val);
}

__global__ void k_um_empty(int32_t* __restrict__ n_unique_miss) {
    if (threadIdx.x < 2) n_unique_miss[threadIdx.x] = 0;
}

// ---- coalescing of the missed rows (Section II-A of the paper) -------------------------------------------
// Instead of one staged row per missed lookup, the distinct missed rows are listed once (ascending gid) and
// every missed lookup's loc points at its row in that list: pairs (gid, miss rank) are sorted by gid, run heads
// are compacted into unique_miss_gid, and each pair writes loc[miss_pos[rank]] = k + (index of its run).
__global__ __launch_bounds__(kBlock) void k_um_prepare(const int32_t* __restrict__ miss_gid, const int32_t* __restrict__ n_hit_miss,
                                                       uint32_t* __restrict__ key, uint32_t* __restrict__ val) {
    const int64_t n = n_hit_miss[1];
    for (int64_t j = (int64_t)blockIdx.x * kBlock + threadIdx.x; j < n; j += (int64_t)gridDim.x * kBlock) {
        key[j] = (uint32_t)miss_gid[j];
        val[j] = (uint32_t)j;
    }
}

__global__ __launch_bounds__(kBlock) void k_um_count(const uint32_t* __restrict__ key, const int32_t* __restrict__ n_hit_miss,
                                                     uint32_t* __restrict__ blk_head, uint32_t* __restrict__ blk_n) {
    __shared__ uint32_t s_a[4], s_b[4];
    const int64_t n = n_hit_miss[1];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + wave_id() * kPerWave;
    uint32_t nh = 0, nv = 0;
#pragma unroll
    for (int r = 0; r < kRoundsR; ++r) {
        const int64_t j = base + r * kWave + lane_id();
        const bool in = j < n;
        const bool head = in && (j == 0 || key[j - 1] != key[j]);
        nh += (uint32_t)__popcll(ballot64(head));
        nv += (uint32_t)__popcll(ballot64(in));
    }
    if (lane_id() == 0) { s_a[wave_id()] = nh; s_b[wave_id()] = nv; }
    __syncthreads();
    if (threadIdx.x == 0) {
        blk_head[blockIdx.x] = s_a[0] + s_a[1] + s_a[2] + s_a[3];
        blk_n[blockIdx.x] = s_b[0] + s_b[1] + s_b[2] + s_b[3];
    }
}

__global__ __launch_bounds__(kBlock) void k_um_write(const uint32_t* __restrict__ key, const uint32_t* __restrict__ val,
                                                     const int32_t* __restrict__ n_hit_miss, const uint32_t* __restrict__ blk_head,
                                                     const uint32_t* __restrict__ blk_n, int scanned,
                                                     int32_t* __restrict__ n_unique_miss, int32_t k,
                                                     const int32_t* __restrict__ miss_pos,
                                                     int32_t* __restrict__ unique_miss_gid, int32_t* __restrict__ loc) {
    __shared__ uint32_t s_a[4], s_red[8];
    const int64_t n = n_hit_miss[1];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + wave_id() * kPerWave;
    uint32_t kk[kRoundsR];
    bool hd[kRoundsR];
    uint32_t nh = 0;
#pragma unroll
    for (int r = 0; r < kRoundsR; ++r) {
        const int64_t j = base + r * kWave + lane_id();
        kk[r] = j < n ? key[j] : 0u;
        hd[r] = j < n && (j == 0 || key[j - 1] != kk[r]);
        nh += (uint32_t)__popcll(ballot64(hd[r]));
    }
    if (lane_id() == 0) s_a[wave_id()] = nh;
    __syncthreads();
    uint32_t before, bn, ta, tb;
    tile_prefix2(blk_head, blk_n, blockIdx.x, gridDim.x, scanned != 0, s_red, n_unique_miss, &before, &bn, &ta, &tb);
    for (int w = 0; w < wave_id(); ++w) before += s_a[w];
#pragma unroll
    for (int r = 0; r < kRoundsR; ++r) {
        const int64_t j = base + r * kWave + lane_id();
        const uint64_t m = ballot64(hd[r]);
        if (j < n) {
            // index of this pair's run = heads at or before j, minus one
            const uint32_t u = before + (uint32_t)rank_below(m) + (hd[r] ? 1u : 0u) - 1u;
            if (hd[r]) unique_miss_gid[u] = (int32_t)kk[r];
            loc[miss_pos[val[j]]] = k + (int32_t)u;
        }
        before += (uint32_t)__popcll(m);
    }
}

hipError_t launch_remap(scars_handle* h, hipStream_t s, const int32_t* idx, const int32_t* off, int64_t L, int64_t B,
                        const scars_remap_out* out) {
    Workspace& ws = h->ws;
    const int nb = (int)std::max<int64_t>(1, div_up(L, kScanTile));
    {
        Timed t(h, s, "remap_probe");
        hipLaunchKernelGGL(k_remap_probe, dim3(nb), dim3(kBlock), 0, s, idx, off, L, B, ws.meta, h->buf.slot_of,
                           out->slot, out->gid, ws.blk_hit, ws.blk_miss, ws.status);
    }
    const bool scan = nb > h->fused_scan_max_tiles;   // few tiles: the writer adds up the tile counts itself
    if (scan) {
        Timed t(h, s, "remap_scan");
        hipLaunchKernelGGL(k_remap_scan, dim3(1), dim3(kBlock), 0, s, ws.blk_hit, ws.blk_miss, nb, out->n_hit_miss);
    }
    // the pairs go into the first sort buffer, which listing each distinct missed row once (below) sorts in as well
    const bool pairs = h->pairs_in_remap && !h->lookahead && L > 0 && !out->unique_miss_gid;
    h->pairs_valid = false;
    if (pairs) {
        Timed t(h, s, "remap_write");
        const int64_t G = (int64_t)h->T * B;
        const int lpb = pairs_lanes_per_bag(L, G);
        const int64_t pair_blocks = div_up(G * lpb, kBlock);
        hipLaunchKernelGGL(k_remap_write_pairs, dim3((unsigned)(nb + pair_blocks)), dim3(kBlock), 0, s, nb, L, out->slot,
                           out->gid, ws.blk_hit, ws.blk_miss, scan ? 1 : 0, out->n_hit_miss, (int32_t)h->k, out->loc,
                           out->hit_pos, out->miss_pos, out->miss_gid, off, G, lpb, bag_shift_host(G), ws.key_buf[0], ws.val_buf[0]);
        h->pairs_valid = true;
        h->pairs_gid = out->gid; h->pairs_off = off; h->pairs_L = L; h->pairs_B = B;
    } else {
        Timed t(h, s, "remap_write");
        hipLaunchKernelGGL(k_remap_write, dim3(nb), dim3(kBlock), 0, s, L, out->slot, out->gid, ws.blk_hit, ws.blk_miss,
                           scan ? 1 : 0, out->n_hit_miss, (int32_t)h->k, out->loc, out->hit_pos, out->miss_pos,
                           out->miss_gid);
    }
    if (out->unique_miss_gid && L > 0 && h->k < h->N) {
        const int grid = (int)std::min<int64_t>(div_up(L, kBlock), 256 * 8);
        {
            Timed t(h, s, "um_prepare");
            hipLaunchKernelGGL(k_um_prepare, dim3(grid), dim3(kBlock), 0, s, out->miss_gid, out->n_hit_miss, ws.key_buf[0],
                               ws.val_buf[0]);
        }
        int bits = 1;
        while (bits < 32 && ((int64_t)1 << bits) < h->N) ++bits;      // gids are below N
        int res = 0;
        hipError_t e = launch_radix_sort_pairs(h, s, ws.key_buf, ws.val_buf, L, out->n_hit_miss + 1, bits, &res);
        if (e != hipSuccess) return e;
        {
            Timed t(h, s, "um_count");
            hipLaunchKernelGGL(k_um_count, dim3(nb), dim3(kBlock), 0, s, ws.key_buf[res], out->n_hit_miss, ws.blk_hit,
                               ws.blk_miss);
        }
        if (scan) {
            Timed t(h, s, "um_scan");
            hipLaunchKernelGGL(k_remap_scan, dim3(1), dim3(kBlock), 0, s, ws.blk_hit, ws.blk_miss, nb, out->n_unique_miss);
        }
        {
            Timed t(h, s, "um_write");
            hipLaunchKernelGGL(k_um_write, dim3(nb), dim3(kBlock), 0, s, ws.key_buf[res], ws.val_buf[res], out->n_hit_miss,
                               ws.blk_hit, ws.blk_miss, scan ? 1 : 0, out->n_unique_miss, (int32_t)h->k, out->miss_pos,
                               out->unique_miss_gid, out->loc);
        }
    } else if (out->unique_miss_gid) {
        Timed t(h, s, "um_empty");   // nothing can miss: the list is empty
        hipLaunchKernelGGL(k_um_empty, dim3(1), dim3(kWave), 0, s, out->n_unique_miss);
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) h->pairs_valid = false;
    return e;
}

// ---- remap with the scratch in the library's own static device array ---------------------------------------
// For callers that cannot hand over (or allocate) a workspace: everything scars_remap keeps in the bound workspace
// for this step -- the table descriptor, the status word, the per-tile hit and miss counts -- lives in one file-scope
// device array instead.  Each GPU holds its own copy of that array at its own address; the address is looked up once
// per device with hipGetSymbolAddress and only that pointer is ever handed to kernels or copies.
constexpr int64_t kStaticMaxTiles = kStaticRemapMaxL / kScanTile;                       // 4096
constexpr int64_t kStaticMetaOff = 0;
constexpr int64_t kStaticStatusOff = (sizeof(Meta) + 255) / 256 * 256;
constexpr int64_t kStaticHitOff = kStaticStatusOff + 256;
constexpr int64_t kStaticTileBytes = ((kStaticMaxTiles + 1) * 4 + 255) / 256 * 256;
constexpr int64_t kStaticMissOff = kStaticHitOff + kStaticTileBytes;
constexpr int64_t kStaticBytes = kStaticMissOff + kStaticTileBytes;
static_assert(kStaticBytes <= 64 * 1024, "the static scratch is meant to stay modest");

static __device__ __align__(256) unsigned char scratch[kStaticBytes];   // zero when the code object is loaded

constexpr int kStaticMaxDevices = 64;
static std::mutex g_static_mu;
static void* g_static_ptr[kStaticMaxDevices];      // per device: address of that device's copy of `scratch`

// Address of the current device's copy of the array (looked up on the first call on that device).
static hipError_t static_scratch(unsigned char** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kStaticMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_static_mu);
    if (!g_static_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_static_ptr[dev] = p;
    }
    *out = (unsigned char*)g_static_ptr[dev];
    return hipSuccess;
}

int32_t* static_status_if_used() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kStaticMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_static_mu);
    return g_static_ptr[dev] ? (int32_t*)((unsigned char*)g_static_ptr[dev] + kStaticStatusOff) : nullptr;
}

// The part of the descriptor the remap kernels read (row_base, num_tables), handed over as kernel arguments: a copy
// from ordinary host memory could make the runtime allocate a staging buffer.
constexpr int kMetaPack = 512;
struct MetaPack { int32_t v[kMetaPack]; };

__global__ void k_static_meta(Meta* __restrict__ meta, int first, int n, int num_tables, MetaPack pack) {
    for (int i = threadIdx.x; i < n; i += blockDim.x) meta->row_base[first + i] = pack.v[i];
    if (threadIdx.x == 0) meta->num_tables = num_tables;
}

hipError_t launch_remap_static(scars_handle* h, hipStream_t s, const int32_t* idx, const int32_t* off, int64_t L, int64_t B,
                               const scars_remap_out* out) {
    unsigned char* base = nullptr;
    hipError_t e = static_scratch(&base);
    if (e != hipSuccess) return e;
    Meta* meta = (Meta*)(base + kStaticMetaOff);
    int32_t* status = (int32_t*)(base + kStaticStatusOff);
    uint32_t* blk_hit = (uint32_t*)(base + kStaticHitOff);
    uint32_t* blk_miss = (uint32_t*)(base + kStaticMissOff);
    // another handle may have used the array last: the descriptor is written again on every call (stream order)
    for (int first = 0; first <= h->T; first += kMetaPack) {
        MetaPack pack;
        const int n = std::min(kMetaPack, h->T + 1 - first);
        for (int i = 0; i < n; ++i) pack.v[i] = (int32_t)h->row_base[first + i];
        Timed t(h, s, "static_meta");
        hipLaunchKernelGGL(k_static_meta, dim3(1), dim3(kBlock), 0, s, meta, first, n, h->T, pack);
    }
    const int nb = (int)std::max<int64_t>(1, div_up(L, kScanTile));     // <= kStaticMaxTiles: the caller checked L
    {
        Timed t(h, s, "remap_probe");
        hipLaunchKernelGGL(k_remap_probe, dim3(nb), dim3(kBlock), 0, s, idx, off, L, B, meta, h->buf.slot_of, out->slot,
                           out->gid, blk_hit, blk_miss, status);
    }
    const bool scan = nb > h->fused_scan_max_tiles;
    if (scan) {
        Timed t(h, s, "remap_scan");
        hipLaunchKernelGGL(k_remap_scan, dim3(1), dim3(kBlock), 0, s, blk_hit, blk_miss, nb, out->n_hit_miss);
    }
    {
        Timed t(h, s, "remap_write");
        hipLaunchKernelGGL(k_remap_write, dim3(nb), dim3(kBlock), 0, s, L, out->slot, out->gid, blk_hit, blk_miss,
                           scan ? 1 : 0, out->n_hit_miss, (int32_t)h->k, out->loc, out->hit_pos, out->miss_pos, out->miss_gid);
    }
    return hipGetLastError();
}

}  // namespace scars
