// build_cache: skew table (occurrence histogram), top-k selection under the row budget, cache fill.
//
// Section III of the paper builds a ranked skew table over all embeddings and keeps the top entries on the
// device; Section IV fixes the cached set by a byte budget.  Here: (1) counts[gid] += 1 per lookup;
// (2) a three-pass most-significant-digit radix select finds the count c* of the k-th row in the order
// (count descending, gid ascending) and how many rows of count c* belong to the top k; (3) an ordered
// compaction lists the winners in ascending gid (all rows above c*, and the lowest-id rows at c*);
// (4) a stable sort by descending count puts them in hotness order, which is the slot order;
// (5) rows are copied from pinned host memory into the cache.
#include "scars_dev.h"

namespace scars {

__global__ __launch_bounds__(kBlock) void k_fill_u32(uint32_t* __restrict__ p, int64_t n, uint32_t v) {
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (int64_t)gridDim.x * kBlock) p[i] = v;
}

hipError_t launch_fill_u32(scars_handle* h, hipStream_t s, uint32_t* p, int64_t n, uint32_t v) {
    if (n <= 0) return hipSuccess;
    Timed t(h, s, "fill_u32");
    int grid = (int)std::min<int64_t>(div_up(n, kBlock), 256 * 16);
    hipLaunchKernelGGL(k_fill_u32, dim3(grid), dim3(kBlock), 0, s, p, n, v);
    return hipGetLastError();
}

// Plain streaming copy of 16-byte words: the known-size kernel against which HBM byte counters are scaled, and the
// box's own copy rate.  Grid-stride with streaming loads and stores, two independent 16-byte loads in flight per lane
// and 16384 workgroups: swept over 2/4/8 loads, 2048 .. 65536 workgroups, cached and streaming accesses, this is the
// fastest (5.3 - 5.4 TB/s on 1 GiB each way, a little above the runtime's own device-to-device copy).
constexpr int kCopyUnroll = 2;
constexpr int kCopyGrid = 16384;
__global__ __launch_bounds__(kBlock) void k_calib_copy(u32x4* __restrict__ dst, const u32x4* __restrict__ src, int64_t n16) {
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    for (; i + (kCopyUnroll - 1) * stride < n16; i += kCopyUnroll * stride) {
        u32x4 v[kCopyUnroll];
#pragma unroll
        for (int u = 0; u < kCopyUnroll; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < kCopyUnroll; ++u) __builtin_nontemporal_store(v[u], dst + i + u * stride);
    }
    for (; i < n16; i += stride) dst[i] = src[i];
}

hipError_t launch_calib_copy(hipStream_t s, void* dst, const void* src, int64_t bytes) {
    const int64_t n16 = bytes / 16;
    if (n16 <= 0) return hipSuccess;
    const unsigned grid = (unsigned)std::min<int64_t>(kCopyGrid, div_up(n16, kBlock));
    hipLaunchKernelGGL(k_calib_copy, dim3(grid), dim3(kBlock), 0, s, (u32x4*)dst, (const u32x4*)src, n16);
    return hipGetLastError();
}

// Host-link calibration: `n` granules of `lpr` 16-byte pieces each move between pinned host memory and a device buffer.
// Granule j of the device buffer pairs with granule pick(j) of the host buffer, pick = a 64-bit mixer of j modulo the
// host buffer's granules (scattered like the rows of a batch) or j itself (sequential).  to_host 0: host -> device,
// the access pattern of the missed-row fetch; 1: device -> host, that of the cold-row write-back.
__device__ __forceinline__ uint64_t mix64(uint64_t x) {
    x += 0x9E3779B97F4A7C15ull;
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    return x ^ (x >> 31);
}

__global__ __launch_bounds__(kBlock) void k_calib_link(u32x4* __restrict__ host, int64_t host_granules, u32x4* __restrict__ dev,
                                                       int64_t n, int lpr, int scattered, int to_host) {
    const int gpb = kBlock / lpr;
    const int grp = threadIdx.x / lpr, gl = threadIdx.x % lpr;
    const int64_t stride = (int64_t)gridDim.x * gpb;
    constexpr int U = 4;
    for (int64_t j0 = (int64_t)blockIdx.x * gpb + grp; j0 < n; j0 += stride * U) {
        int64_t hj[U];
        u32x4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t j = min(j0 + u * stride, n - 1);
            hj[u] = scattered ? (int64_t)(mix64((uint64_t)j) % (uint64_t)host_granules) : j % host_granules;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t j = min(j0 + u * stride, n - 1);
            v[u] = to_host ? dev[j * lpr + gl] : __builtin_nontemporal_load(host + hj[u] * lpr + gl);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t j = j0 + u * stride;
            if (j < n) {
                if (to_host) host[hj[u] * lpr + gl] = v[u]; else dev[j * lpr + gl] = v[u];
            }
        }
    }
}

hipError_t launch_calib_link(hipStream_t s, void* host, int64_t host_bytes, void* dev, int64_t n, int granule_bytes,
                             int scattered, int to_host, int blocks) {
    const int lpr = granule_bytes / 16;
    hipLaunchKernelGGL(k_calib_link, dim3(blocks), dim3(kBlock), 0, s, (u32x4*)host, host_bytes / granule_bytes, (u32x4*)dev, n,
                       lpr, scattered, to_host);
    return hipGetLastError();
}

// Plain streaming read: every 16-byte word is loaded once and folded into one word per thread (written to `sink`,
// gridDim * kBlock words), so the box's read-only rate can stand beside the copy rate.
constexpr int kCalibReadGrid = 256 * 16;
__global__ __launch_bounds__(kBlock) void k_calib_read(const u32x4* __restrict__ src, int64_t n16, uint32_t* __restrict__ sink) {
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    u32x4 acc = {0u, 0u, 0u, 0u};
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const u32x4 a = __builtin_nontemporal_load(src + i), b = __builtin_nontemporal_load(src + i + stride);
        const u32x4 c = __builtin_nontemporal_load(src + i + 2 * stride), d = __builtin_nontemporal_load(src + i + 3 * stride);
        acc ^= a ^ b ^ c ^ d;
    }
    for (; i < n16; i += stride) acc ^= __builtin_nontemporal_load(src + i);
    sink[(int64_t)blockIdx.x * kBlock + threadIdx.x] = acc.x ^ acc.y ^ acc.z ^ acc.w;
}

hipError_t launch_calib_read(hipStream_t s, const void* src, int64_t bytes, void* sink) {
    hipLaunchKernelGGL(k_calib_read, dim3(kCalibReadGrid), dim3(kBlock), 0, s, (const u32x4*)src, bytes / 16, (uint32_t*)sink);
    return hipGetLastError();
}

// ---- (1) histogram --------------------------------------------------------------------------------
// The table of a lookup follows from its position: lookups of table t occupy [offsets[t*B], offsets[(t+1)*B]).
// A workgroup takes kHistChunk consecutive lookups and first adds them up in an LDS table keyed by row id (open
// addressing, at most half full), then issues one global atomic per distinct row of its chunk: under skew the hot
// rows, which would otherwise serialise thousands of atomics on one address, arrive as a few hundred sums.
constexpr int kHistChunk = 2048;            // lookups per workgroup
constexpr int kHistSlots = 2 * kHistChunk;  // LDS table slots (power of two)
constexpr uint32_t kHistEmpty = 0xFFFFFFFFu;

__global__ __launch_bounds__(kBlock) void k_histogram(const int32_t* __restrict__ idx, const int32_t* __restrict__ off,
                                                      int64_t L, int64_t B, const Meta* __restrict__ meta,
                                                      uint32_t* __restrict__ counts, int32_t* __restrict__ status) {
    __shared__ int32_t s_tstart[SCARS_MAX_TABLES + 1];
    __shared__ int32_t s_rbase[SCARS_MAX_TABLES + 1];
    __shared__ uint32_t s_key[kHistSlots];
    __shared__ uint32_t s_cnt[kHistSlots];
    const int T = meta->num_tables;
    for (int t = threadIdx.x; t <= T; t += kBlock) {
        s_tstart[t] = off[(int64_t)t * B];
        s_rbase[t] = meta->row_base[t];
    }
    for (int i = threadIdx.x; i < kHistSlots; i += kBlock) { s_key[i] = kHistEmpty; s_cnt[i] = 0u; }
    __syncthreads();
    const int64_t G = (int64_t)T * B;
    const int64_t nthreads = (int64_t)gridDim.x * kBlock;
    const int64_t gt = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    // offsets must start at 0, end at L and never decrease
    for (int64_t g = gt; g < G; g += nthreads)
        if (off[g + 1] < off[g]) latch_error(status, SCARS_ERR_OFFSETS);
    if (gt == 0 && (off[0] != 0 || (int64_t)off[G] != L)) latch_error(status, SCARS_ERR_OFFSETS);
    const int64_t c0 = (int64_t)blockIdx.x * kHistChunk;
    constexpr int kPer = kHistChunk / kBlock;
    int32_t r[kPer];
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
        const int64_t i = c0 + (int64_t)u * kBlock + threadIdx.x;
        r[u] = i < L ? idx[i] : 0;
    }
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
        const int64_t i = c0 + (int64_t)u * kBlock + threadIdx.x;
        if (i >= L) continue;
        const int t = upper_table(s_tstart, T, (int32_t)i);
        const int32_t nrows = s_rbase[t + 1] - s_rbase[t];
        if (r[u] < 0 || r[u] >= nrows) {
            latch_error(status, SCARS_ERR_INDEX_RANGE);
            continue;
        }
        const uint32_t gid = (uint32_t)(s_rbase[t] + r[u]);     // below 2^31: never the empty mark
        uint32_t h = (gid * 0x9E3779B1u) >> (32 - 12);           // kHistSlots = 2^12
        for (int probe = 0; probe < kHistSlots; ++probe) {       // the table is at most half full: an empty slot exists
            const uint32_t prev = atomicCAS(&s_key[h], kHistEmpty, gid);
            if (prev == kHistEmpty || prev == gid) {
                atomicAdd(&s_cnt[h], 1u);
                break;
            }
            h = (h + 1) & (kHistSlots - 1);
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kHistSlots; i += kBlock) {
        const uint32_t c = s_cnt[i];
        if (c) atomicAdd(&counts[s_key[i]], c);
    }
}
static_assert(kHistSlots == (1 << 12), "the hash above keeps 12 bits");

hipError_t launch_histogram(scars_handle* h, hipStream_t s, const int32_t* idx, const int32_t* off, int64_t L,
                            int64_t B) {
    Timed t(h, s, "histogram");
    // enough workgroups for the lookups (a chunk each) and, in their grid-stride loop, for the offsets check
    const int64_t grid = std::max<int64_t>(1, div_up(L, kHistChunk));
    hipLaunchKernelGGL(k_histogram, dim3((unsigned)grid), dim3(kBlock), 0, s, idx, off, L, B, h->ws.meta, h->buf.counts,
                       h->ws.status);
    return hipGetLastError();
}

// ---- (2) radix select over the counts, most significant digit first ---------------------------------
// sel_state[0] = decided high bits of c*, sel_state[1] = rows still to take from the undecided bucket.
__device__ __forceinline__ void sel_pass_bits(int pass, int* shift, uint32_t* nbins) {
    // 32 bits = 11 + 11 + 10
    if (pass == 0) { *shift = 21; *nbins = 2048; }
    else if (pass == 1) { *shift = 10; *nbins = 2048; }
    else { *shift = 0; *nbins = 1024; }
}

__global__ __launch_bounds__(kBlock) void k_sel_init(uint32_t* __restrict__ sel_state, uint32_t* __restrict__ sel_hist,
                                                     uint32_t k) {
    for (int i = threadIdx.x; i < 3 * kSelBins; i += kBlock) sel_hist[i] = 0;
    if (threadIdx.x == 0) { sel_state[0] = 0; sel_state[1] = k; }
}

__global__ __launch_bounds__(kBlock) void k_sel_hist(const uint32_t* __restrict__ counts, int64_t N, int pass,
                                                     const uint32_t* __restrict__ sel_state, uint32_t* __restrict__ hist) {
    __shared__ uint32_t s_h[kSelBins];
    for (int i = threadIdx.x; i < kSelBins; i += kBlock) s_h[i] = 0;
    __syncthreads();
    int shift; uint32_t nbins;
    sel_pass_bits(pass, &shift, &nbins);
    const uint32_t prefix = sel_state[0];
    const int hi_shift = pass == 0 ? 32 : (pass == 1 ? 21 : 10);   // bits above are already decided
    for (int64_t base = (int64_t)blockIdx.x * kBlock; base < N; base += (int64_t)gridDim.x * kBlock) {
        const int64_t g = base + threadIdx.x;
        bool in = g < N;
        uint32_t c = in ? counts[g] : 0u;
        if (in && pass > 0) in = (c >> hi_shift) == (prefix >> hi_shift);
        const uint32_t d = (c >> shift) & (nbins - 1);
        // most rows share one digit (count 0 or 1): one LDS atomic per wave in that case
        const uint64_t act = ballot64(in);
        if (act) {
            const int leader = __ffsll((unsigned long long)act) - 1;
            const uint32_t d0 = __shfl(d, leader, 64);
            const uint64_t same = ballot64(in && d == d0);
            if (same == act) {
                if (lane_id() == leader) atomicAdd(&s_h[d0], (uint32_t)__popcll(act));
            } else if (in) {
                atomicAdd(&s_h[d], 1u);
            }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < (int)nbins; i += kBlock)
        if (s_h[i]) atomicAdd(&hist[pass * kSelBins + i], s_h[i]);
}

// single workgroup: walk the bins from the largest digit down until the remaining quota is met
__global__ __launch_bounds__(kBlock) void k_sel_pick(int pass, uint32_t* __restrict__ sel_state,
                                                     const uint32_t* __restrict__ hist) {
    __shared__ uint32_t s_scan[8];
    __shared__ uint32_t s_found[2];
    int shift; uint32_t nbins;
    sel_pass_bits(pass, &shift, &nbins);
    const uint32_t krem = sel_state[1];
    if (threadIdx.x == 0) { s_found[0] = 0xFFFFFFFFu; s_found[1] = 0; }
    __syncthreads();
    // descending bin order: position j <-> bin nbins-1-j; find first j with inclusive cumulative >= krem
    uint32_t carry = 0;
    for (uint32_t base = 0; base < nbins; base += kBlock) {
        const uint32_t j = base + threadIdx.x;
        const uint32_t v = hist[pass * kSelBins + (nbins - 1 - j)];
        uint32_t total;
        const uint32_t ex = carry + block_exclusive_scan(v, s_scan, &total);
        if (ex < krem && ex + v >= krem) { s_found[0] = nbins - 1 - j; s_found[1] = ex; }
        carry += total;
        __syncthreads();
    }
    if (threadIdx.x == 0 && s_found[0] != 0xFFFFFFFFu) {
        sel_state[0] |= s_found[0] << shift;
        sel_state[1] = krem - s_found[1];
    }
}

// ---- (3) ordered compaction of the winners ----------------------------------------------------------
// Tile of kScanTile gids per workgroup; each wave owns kScanTile/4 consecutive gids in 8 rounds of 64.
constexpr int kScanPerWave = kScanTile / (kBlock / kWave);   // 512
constexpr int kScanRounds = kScanPerWave / kWave;            // 8

__global__ __launch_bounds__(kBlock) void k_win_count(const uint32_t* __restrict__ counts, int64_t N,
                                                      const uint32_t* __restrict__ sel_state,
                                                      uint32_t* __restrict__ blk_gt, uint32_t* __restrict__ blk_eq) {
    __shared__ uint32_t s_gt[4], s_eq[4];
    const uint32_t cstar = sel_state[0];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + wave_id() * kScanPerWave;
    uint32_t ngt = 0, neq = 0;
#pragma unroll
    for (int r = 0; r < kScanRounds; ++r) {
        const int64_t g = base + r * kWave + lane_id();
        const uint32_t c = g < N ? counts[g] : 0u;
        ngt += (uint32_t)__popcll(ballot64(g < N && c > cstar));
        neq += (uint32_t)__popcll(ballot64(g < N && c == cstar));
    }
    if (lane_id() == 0) { s_gt[wave_id()] = ngt; s_eq[wave_id()] = neq; }
    __syncthreads();
    if (threadIdx.x == 0) {
        blk_gt[blockIdx.x] = s_gt[0] + s_gt[1] + s_gt[2] + s_gt[3];
        blk_eq[blockIdx.x] = s_eq[0] + s_eq[1] + s_eq[2] + s_eq[3];
    }
}

// single workgroup: exclusive scan in place of two arrays of n entries; totals to a[n], b[n]
__global__ __launch_bounds__(kBlock) void k_scan_two(uint32_t* __restrict__ a, uint32_t* __restrict__ b, int n) {
    __shared__ uint32_t s_scan[8];
    uint32_t ca, cb;
    scan_two_counts(a, b, n, s_scan, &ca, &cb);
    if (threadIdx.x == 0) { a[n] = ca; b[n] = cb; }
}

__global__ __launch_bounds__(kBlock) void k_win_write(const uint32_t* __restrict__ counts, int64_t N,
                                                      const uint32_t* __restrict__ sel_state,
                                                      const uint32_t* __restrict__ blk_gt, const uint32_t* __restrict__ blk_eq,
                                                      uint32_t* __restrict__ win_key, uint32_t* __restrict__ win_gid,
                                                      int32_t* __restrict__ slot_of, uint32_t k) {
    __shared__ uint32_t s_gt[4], s_eq[4];
    const uint32_t cstar = sel_state[0], need = sel_state[1];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + wave_id() * kScanPerWave;
    uint32_t c[kScanRounds];
    uint32_t ngt = 0, neq = 0;
#pragma unroll
    for (int r = 0; r < kScanRounds; ++r) {
        const int64_t g = base + r * kWave + lane_id();
        c[r] = g < N ? counts[g] : 0u;
        ngt += (uint32_t)__popcll(ballot64(g < N && c[r] > cstar));
        neq += (uint32_t)__popcll(ballot64(g < N && c[r] == cstar));
    }
    if (lane_id() == 0) { s_gt[wave_id()] = ngt; s_eq[wave_id()] = neq; }
    __syncthreads();
    uint32_t gt_before = blk_gt[blockIdx.x], eq_before = blk_eq[blockIdx.x];
    for (int w = 0; w < wave_id(); ++w) { gt_before += s_gt[w]; eq_before += s_eq[w]; }
#pragma unroll
    for (int r = 0; r < kScanRounds; ++r) {
        const int64_t g = base + r * kWave + lane_id();
        const bool in = g < N;
        const bool gt = in && c[r] > cstar, eq = in && c[r] == cstar;
        const uint64_t mgt = ballot64(gt), meq = ballot64(eq);
        const uint32_t my_gt = gt_before + (uint32_t)rank_below(mgt);
        const uint32_t my_eq = eq_before + (uint32_t)rank_below(meq);
        const bool win = k > 0 && (gt || (eq && my_eq < need));
        if (in) slot_of[g] = -1;
        if (win) {
            const uint32_t pos = my_gt + min(my_eq, need);
            win_key[pos] = ~c[r];
            win_gid[pos] = (uint32_t)g;
        }
        gt_before += (uint32_t)__popcll(mgt);
        eq_before += (uint32_t)__popcll(meq);
    }
}

// ---- (4)/(5) slots and cache fill ---------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void k_slot_scatter(const uint32_t* __restrict__ sorted_gid, int64_t k,
                                                         int32_t* __restrict__ hot_gid, int32_t* __restrict__ slot_of) {
    const int64_t s = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (s < k) {
        const int32_t g = (int32_t)sorted_gid[s];
        hot_gid[s] = g;
        slot_of[g] = (int32_t)s;
    }
}

// Copy rows between pinned host tables and the cache, `lpr` lanes per row, 16 bytes per lane per step.
// to_cache: host -> cache; else cache -> host.  `chunks` = 16-byte pieces per row.
__global__ __launch_bounds__(kBlock) void k_cache_copy(const int32_t* __restrict__ hot_gid, int64_t k,
                                                       const Meta* __restrict__ meta, uint4* __restrict__ cache,
                                                       int chunks, int lpr, int to_cache, int with_state,
                                                       uint4* __restrict__ state_cache, int state_chunks) {
    __shared__ int32_t s_rbase[SCARS_MAX_TABLES + 1];
    const int T = meta->num_tables;
    for (int t = threadIdx.x; t <= T; t += kBlock) s_rbase[t] = meta->row_base[t];
    __syncthreads();
    const int groups_per_block = kBlock / lpr;
    const int grp = threadIdx.x / lpr, gl = threadIdx.x % lpr;
    for (int64_t s = (int64_t)blockIdx.x * groups_per_block + grp; s < k; s += (int64_t)gridDim.x * groups_per_block) {
        const int32_t gid = hot_gid[s];
        const int t = upper_table(s_rbase, T, gid);
        const int64_t row = gid - s_rbase[t];
        uint4* host = (uint4*)meta->table[t] + row * chunks;
        uint4* dev = cache + s * chunks;
        for (int c = gl; c < chunks; c += lpr) {
            if (to_cache) dev[c] = host[c]; else host[c] = dev[c];
        }
        if (with_state) {
            uint4* hs = (uint4*)meta->state[t] + row * state_chunks;
            uint4* ds = state_cache + s * state_chunks;
            for (int c = gl; c < state_chunks; c += lpr) {
                if (to_cache) ds[c] = hs[c]; else hs[c] = ds[c];
            }
        }
    }
}

static hipError_t launch_cache_copy(scars_handle* h, hipStream_t s, int to_cache, const char* name) {
    if (h->k <= 0) return hipSuccess;
    Timed t(h, s, name);
    const int chunks = h->R / 16;
    const int lpr = std::min(64, next_pow2_host(chunks));
    const int with_state = h->optimizer == SCARS_OPT_ADAGRAD;
    const int gpb = kBlock / lpr;
    int grid = (int)std::min<int64_t>(div_up(h->k, gpb), 256 * 32);
    hipLaunchKernelGGL(k_cache_copy, dim3(grid), dim3(kBlock), 0, s, h->buf.hot_gid, h->k, h->ws.meta,
                       (uint4*)h->buf.cache, chunks, lpr, to_cache, with_state, (uint4*)h->buf.state_cache,
                       h->D * 4 / 16);
    return hipGetLastError();
}

hipError_t launch_flush(scars_handle* h, hipStream_t s) { return launch_cache_copy(h, s, 0, "cache_flush"); }

hipError_t launch_select_and_fill(scars_handle* h, hipStream_t s, int64_t k) {
    const int64_t N = h->N;
    Workspace& ws = h->ws;
    const int nbN = (int)div_up(N, kScanTile);
    {
        Timed t(h, s, "sel_init");
        hipLaunchKernelGGL(k_sel_init, dim3(1), dim3(kBlock), 0, s, ws.sel_state, ws.sel_hist, (uint32_t)k);
    }
    if (k > 0) {
        const int grid = (int)std::min<int64_t>(div_up(N, kBlock), 256 * 16);
        for (int pass = 0; pass < 3; ++pass) {
            {
                Timed t(h, s, "sel_hist");
                hipLaunchKernelGGL(k_sel_hist, dim3(grid), dim3(kBlock), 0, s, h->buf.counts, N, pass, ws.sel_state,
                                   ws.sel_hist);
            }
            {
                Timed t(h, s, "sel_pick");
                hipLaunchKernelGGL(k_sel_pick, dim3(1), dim3(kBlock), 0, s, pass, ws.sel_state, ws.sel_hist);
            }
        }
        {
            Timed t(h, s, "win_count");
            hipLaunchKernelGGL(k_win_count, dim3(nbN), dim3(kBlock), 0, s, h->buf.counts, N, ws.sel_state, ws.blk_gt,
                               ws.blk_eq);
        }
        {
            Timed t(h, s, "scan_two");
            hipLaunchKernelGGL(k_scan_two, dim3(1), dim3(kBlock), 0, s, ws.blk_gt, ws.blk_eq, nbN);
        }
    }
    {
        // with k == 0 this only clears slot_of (sel_state = {0, 0}: nothing wins)
        Timed t(h, s, "win_write");
        hipLaunchKernelGGL(k_win_write, dim3(nbN), dim3(kBlock), 0, s, h->buf.counts, N, ws.sel_state, ws.blk_gt,
                           ws.blk_eq, ws.win_key[0], (uint32_t*)ws.win_gid[0], h->buf.slot_of, (uint32_t)k);
    }
    if (k > 0) {
        uint32_t* keys[2] = {ws.win_key[0], ws.win_key[1]};
        uint32_t* vals[2] = {(uint32_t*)ws.win_gid[0], (uint32_t*)ws.win_gid[1]};
        int res = 0;
        hipError_t e = launch_radix_sort_pairs(h, s, keys, vals, k, nullptr, 32, &res);
        if (e != hipSuccess) return e;
        {
            Timed t(h, s, "slot_scatter");
            hipLaunchKernelGGL(k_slot_scatter, dim3((unsigned)div_up(k, kBlock)), dim3(kBlock), 0, s, vals[res], k,
                               h->buf.hot_gid, h->buf.slot_of);
        }
    }
    h->k = k;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_cache_copy(h, s, 1, "cache_fill");
}

}  // namespace scars
