// Device-side helpers for gfx950 (wave64): ballots, scans, table search, bf16 conversion, status latch.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "scars_internal.h"

namespace scars {

// 16 raw bytes as a native vector (stays in registers; HIP's uint4 struct sometimes lands in scratch)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }
__device__ __forceinline__ int wave_id() { return threadIdx.x >> 6; }

__device__ __forceinline__ uint64_t ballot64(bool p) { return __ballot(p); }

// number of set bits of m strictly below this lane
__device__ __forceinline__ int rank_below(uint64_t m) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0));
}

// inclusive scan of one value per lane across the wave
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
    const int l = lane_id();
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint32_t o = __shfl_up(v, d, 64);
        if (l >= d) v += o;
    }
    return v;
}

// Exclusive scan over the 256 threads of a block; *total receives the block sum. `s` is LDS scratch [8].
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* s, uint32_t* total) {
    uint32_t inc = wave_inclusive_scan(v);
    if (lane_id() == 63) s[wave_id()] = inc;
    __syncthreads();
    uint32_t base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kBlock / kWave; ++w) {
        uint32_t t = s[w];
        if (w < wave_id()) base += t;
        tot += t;
    }
    __syncthreads();
    *total = tot;
    return base + inc - v;
}

// One workgroup: exclusive scan of a[0..n) and b[0..n) in place; the two sums to *ta, *tb.  Thread t owns the items
// [t * per, (t + 1) * per): it adds them up (loads eight at a time), one scan across the threads gives its start, then
// it writes the running sums.  Three steps whatever n is.  s_scan is LDS scratch [8]; every thread must call.
__device__ __forceinline__ void scan_two_counts(uint32_t* __restrict__ a, uint32_t* __restrict__ b, int n, uint32_t* s_scan,
                                                uint32_t* ta, uint32_t* tb) {
    constexpr int kU = 8;
    const int per = (n + kBlock - 1) / kBlock;
    const int i0 = min((int)threadIdx.x * per, n), i1 = min(i0 + per, n);
    uint32_t sa = 0, sb = 0;
    for (int i = i0; i < i1; i += kU) {
        uint32_t va[kU], vb[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int j = min(i + u, i1 - 1);
            va[u] = a[j];
            vb[u] = b[j];
        }
#pragma unroll
        for (int u = 0; u < kU; ++u)
            if (i + u < i1) { sa += va[u]; sb += vb[u]; }
    }
    uint32_t ea = block_exclusive_scan(sa, s_scan, ta);
    uint32_t eb = block_exclusive_scan(sb, s_scan, tb);
    for (int i = i0; i < i1; i += kU) {
        uint32_t va[kU], vb[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int j = min(i + u, i1 - 1);
            va[u] = a[j];
            vb[u] = b[j];
        }
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            if (i + u < i1) {
                a[i + u] = ea;
                b[i + u] = eb;
                ea += va[u];
                eb += vb[u];
            }
        }
    }
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}

// Start of tile t in a two-list compaction, from the per-tile counts a[], b[] of nt tiles.  With `scanned` a scan
// kernel has already turned the counts into exclusive prefixes (and written the totals).  Otherwise the counts are
// raw: the workgroup adds up the tiles before its own (a few loads per thread while nt is small; the host picks the
// scan kernel beyond that), and the workgroup of the last tile also writes the two totals to n_out[0..1].
// Every thread of the workgroup must call; s_red is LDS scratch [8].  Returns true in that last workgroup, with the
// totals in *ta, *tb.
__device__ __forceinline__ bool tile_prefix2(const uint32_t* __restrict__ a, const uint32_t* __restrict__ b, int t, int nt,
                                             bool scanned, uint32_t* s_red, int32_t* __restrict__ n_out, uint32_t* pa,
                                             uint32_t* pb, uint32_t* ta, uint32_t* tb) {
    if (scanned) {
        *pa = a[t];
        *pb = b[t];
        return false;
    }
    uint32_t sa = 0, sb = 0;
    for (int i = threadIdx.x; i < t; i += kBlock) {
        sa += a[i];
        sb += b[i];
    }
    sa = wave_sum(sa);
    sb = wave_sum(sb);
    if (lane_id() == 0) {
        s_red[wave_id()] = sa;
        s_red[4 + wave_id()] = sb;
    }
    __syncthreads();
    sa = s_red[0] + s_red[1] + s_red[2] + s_red[3];
    sb = s_red[4] + s_red[5] + s_red[6] + s_red[7];
    __syncthreads();
    *pa = sa;
    *pb = sb;
    if (t != nt - 1) return false;
    *ta = sa + a[t];
    *tb = sb + b[t];
    if (threadIdx.x == 0 && n_out) {
        n_out[0] = (int32_t)*ta;
        n_out[1] = (int32_t)*tb;
    }
    return true;
}

__device__ __forceinline__ void latch_error(int32_t* status, int32_t code) {
    // status[0] holds the first error seen (0 = none); codes are negative
    atomicCAS(status, 0, code);
}

// Largest t in [0, T) with a[t] <= x, for a non-decreasing a[0..T]; clamped so the result is always valid.
__device__ __forceinline__ int upper_table(const int32_t* a, int T, int32_t x) {
    int lo = 0, hi = T;  // answer in [lo, hi)
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (a[mid] <= x) lo = mid; else hi = mid;
    }
    return lo;
}

// (gid, bag) pairs of a batch in position order: key = gid of the lookup (-1, an invalid lookup, becomes the largest
// key), value = (bag << shift) | (place of the lookup inside its bag, saturating at 2^shift - 1).  The place costs
// nothing to carry through the sort and lets the backward pass find a run's first lookup, hence the staged copy of a
// cold row, without searching the bag; `shift` = 32 - (bits of the largest bag id), see bag_shift_host.  A group of
// lpb lanes walks one bag's positions, so the bag id needs no search.  `block` of the workgroups that share this job.
__device__ __forceinline__ void bag_pairs(int64_t block, const int32_t* __restrict__ gid, const int32_t* __restrict__ off,
                                          int32_t L, int64_t G, int lpb, int shift, uint32_t* __restrict__ key,
                                          uint32_t* __restrict__ val) {
    const int64_t g = (block * kBlock + threadIdx.x) / lpb;
    const int c = threadIdx.x % lpb;
    if (g >= G) return;
    const int32_t a = min(max(off[g], 0), L);
    const int32_t b = min(max(off[g + 1], a), L);
    const uint32_t sat = (1u << shift) - 1u;
    for (int32_t i = a + c; i < b; i += lpb) {
        key[i] = (uint32_t)gid[i];
        val[i] = ((uint32_t)g << shift) | min((uint32_t)(i - a), sat);
    }
}

// The piece of a table-major batch that belongs to table t: positions [*a_out, *a_out + *n_out), clamped so that it
// stays inside the batch and within what the per-table sort takes; *over: more lookups than the caller stated.
__device__ __forceinline__ void small_piece(const int32_t* __restrict__ off, int64_t B, int32_t L, int t, int limit,
                                            int32_t* a_out, int32_t* n_out, bool* over) {
    const int32_t a = min(max(off[(int64_t)t * B], 0), L);
    const int32_t b = min(max(off[(int64_t)(t + 1) * B], a), L);
    *over = b - a > limit;
    *a_out = a;
    *n_out = min(b - a, min(limit, kSmallSortCap));
}

// What the update of a small batch needs of its runs, written by the workgroup that sorted the table, at the position
// of each run's first pair in the sorted pieces (run_len null: not wanted): the run's length (0 at every other
// position of the batch) and where its row is found (cache slot, k + row of the staging area, or -1: host memory).
struct SmallRunArgs {
    int32_t *run_len, *run_src;     // [L] each
    const int32_t* loc_of;          // remap's per-lookup locations: cache slot, or k + the lookup's place among the misses
    int32_t k;
    int staged;                     // the missed rows of this batch are in the staging area (else they are read from host memory)
};

struct SmallSortArgs {
    const uint32_t *kin, *vin;      // the batch's (row, value) pairs in position order
    const int32_t* off;
    int64_t B;
    int32_t L;
    int limit;                      // lookups per table the caller stated (<= kSmallSortCap)
    uint32_t *kout, *vout;          // each table's sorted piece, at the piece's own positions
    uint32_t *tab_valid, *tab_heads;   // [T] each: the piece's valid pairs and distinct rows
    int32_t* status;
    SmallRunArgs run;
};

inline SmallSortArgs small_sort_args(const scars_handle* h, uint32_t* const key[2], uint32_t* const val[2], const int32_t* off,
                                     int64_t L, int64_t B) {
    // (the tables' counts take 2 T words of the sort's count matrix, which has kSortMaxBins at least)
    return SmallSortArgs{key[0], val[0], off, B, (int32_t)L, (int)h->table_lookups_limit, key[1], val[1],
                         h->ws.sort_hist, h->ws.sort_hist + h->T, h->ws.status, SmallRunArgs{}};
}

// The run outputs go to the workspace's own run arrays: seg_start as the lengths, unique_slot as the sources.
inline SmallRunArgs small_run_args(const scars_handle* h, const scars_remap_out* rm, bool staged) {
    return SmallRunArgs{h->ws.seg_start, h->ws.unique_slot, rm->loc, (int32_t)h->k, staged ? 1 : 0};
}

// Table t's piece, by the calling workgroup (every thread must call).
__device__ __forceinline__ void small_sort_body(int t, const Meta* __restrict__ meta, const SmallSortArgs& S) {
    constexpr int R = kSmallSortCap / kBlock, kTile = kSmallSortCap;
    constexpr int kMaxBins = kSortMaxBins, kWaves = kBlock / kWave;
    const uint32_t* __restrict__ kin = S.kin;
    const uint32_t* __restrict__ vin = S.vin;
    const int32_t* __restrict__ off = S.off;
    const int64_t B = S.B;
    const int32_t L = S.L;
    const int limit = S.limit;
    uint32_t* __restrict__ kout = S.kout;
    uint32_t* __restrict__ vout = S.vout;
    uint32_t* __restrict__ tab_valid = S.tab_valid;
    uint32_t* __restrict__ tab_heads = S.tab_heads;
    int32_t* __restrict__ status = S.status;
    __shared__ __align__(8) uint32_t s_pairs[2 * kTile];   // the ordered piece; during ranking, the lane sets per wave and digit
    uint32_t* const s_key = s_pairs;
    uint32_t* const s_val = s_pairs + kTile;
    __shared__ uint32_t s_wh[kWaves * kMaxBins];
    __shared__ uint32_t s_dstart[kMaxBins];
    __shared__ uint32_t s_scan[8];
    __shared__ int32_t s_loc[kTile];      // with the run outputs: each pair's location, carried along with the pair
    const bool want_runs = S.run.run_len != nullptr;      // (the same for the whole launch)
    const int tid = threadIdx.x, lane = lane_id(), w = wave_id();
    int32_t a, n;
    bool over;
    small_piece(off, B, L, t, limit, &a, &n, &over);
    if (over && tid == 0) latch_error(status, SCARS_ERR_OFFSETS);   // more lookups in a table than the caller stated
    // the piece is dealt out evenly: wave w owns positions [w * per_wave, (w + 1) * per_wave) in `rounds` rounds of 64
    const int rounds = (n + kBlock - 1) / kBlock;            // <= R
    const int per_wave = rounds * kWave;
    const uint32_t rbase = (uint32_t)meta->row_base[t];
    const uint32_t rows = (uint32_t)meta->row_base[t + 1] - rbase;
    int bits = 1;
    while (bits < 32 && (1u << bits) <= rows) ++bits;      // 2^bits - 1 >= rows: the key of an invalid lookup stays the largest
    const int passes = (bits + 8) / 9;
    const int dbits = (bits + passes - 1) / passes;
    const int bins = 1 << dbits;
    const uint32_t mask = (uint32_t)bins - 1u;

    uint32_t key[R], val[R];
    int32_t lc[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int p = w * per_wave + r * kWave + lane;
        const bool valid = r < rounds && p < n;
        const uint32_t k = valid ? kin[a + p] : 0xFFFFFFFFu;
        key[r] = k == 0xFFFFFFFFu ? k : k - rbase;
        val[r] = valid ? vin[a + p] : 0u;
        lc[r] = (valid && want_runs) ? S.run.loc_of[a + p] : -1;     // (the pair at position a + p is lookup a + p)
    }
    uint32_t* wh = s_wh + w * kMaxBins;
    unsigned long long* const mk = (unsigned long long*)s_pairs + w * kMaxBins;
    for (int pass = 0; pass < passes; ++pass) {
        const int shift = pass * dbits;
        for (int i = tid; i < kWaves * kMaxBins; i += kBlock) s_wh[i] = 0;
        for (int i = tid; i < 2 * kWaves * kMaxBins; i += kBlock) s_pairs[i] = 0;
        __syncthreads();
        // stable rank of every pair among its wave's pairs of the same digit (as in k_sort_scatter; the word of a digit is
        // read and cleared with atomic accesses: the wave's LDS operations on it are carried out in program order)
        uint32_t loc[R], old[R];
        int lead[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            loc[r] = old[r] = 0u;
            lead[r] = 0;
            if (r >= rounds) continue;                       // (the same for every lane of the workgroup)
            const int p = w * per_wave + r * kWave + lane;
            const bool valid = p < n;
            const uint32_t d = (key[r] >> shift) & mask;
            if (valid) atomicOr(&mk[d], 1ull << lane);
            __builtin_amdgcn_wave_barrier();
            const uint64_t m = valid ? __hip_atomic_load(&mk[d], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) : (1ull << lane);
            __builtin_amdgcn_wave_barrier();
            const int rk = rank_below(m);
            lead[r] = __ffsll((unsigned long long)m) - 1;
            loc[r] = (uint32_t)rk;
            old[r] = 0u;
            if (valid && rk == 0) {
                __hip_atomic_store(&mk[d], 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                old[r] = atomicAdd(&wh[d], (uint32_t)__popcll(m));
            }
            __builtin_amdgcn_wave_barrier();
        }
#pragma unroll
        for (int r = 0; r < R; ++r) loc[r] += __shfl(old[r], lead[r], kWave);
        __syncthreads();
        {   // per digit: wave counts -> exclusive wave bases; the piece's count of the digit -> its first position
            uint32_t carry = 0;
            for (int base = 0; base < bins; base += kBlock) {
                const int d = base + tid;
                uint32_t run = 0;
                if (d < bins) {
#pragma unroll
                    for (int ww = 0; ww < kWaves; ++ww) {
                        const uint32_t c = s_wh[ww * kMaxBins + d];
                        s_wh[ww * kMaxBins + d] = run;
                        run += c;
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
        for (int r = 0; r < R; ++r) {
            const int p = w * per_wave + r * kWave + lane;
            if (r < rounds && p < n) {
                const uint32_t d = (key[r] >> shift) & mask;
                const uint32_t q = s_dstart[d] + s_wh[w * kMaxBins + d] + loc[r];
                s_key[q] = key[r];
                s_val[q] = val[r];
                if (want_runs) s_loc[q] = lc[r];
            }
        }
        __syncthreads();
        if (pass + 1 < passes) {   // the ordered piece back into registers, in position order, for the next digit
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int p = w * per_wave + r * kWave + lane;
                if (r < rounds && p < n) {
                    key[r] = s_key[p];
                    val[r] = s_val[p];
                    if (want_runs) lc[r] = s_loc[p];
                }
            }
            __syncthreads();
        }
    }
    uint32_t nv = 0, nh = 0;     // valid pairs; distinct rows among them
    for (int q = tid; q < n; q += kBlock) {
        const uint32_t k = s_key[q];
        const bool ok = k != 0xFFFFFFFFu;
        kout[a + q] = ok ? k + rbase : k;
        vout[a + q] = s_val[q];
        nv += ok ? 1u : 0u;
        nh += (ok && (q == 0 || s_key[q - 1] != k)) ? 1u : 0u;
    }
    nv = wave_sum(nv);
    nh = wave_sum(nh);
    if (lane == 0) { s_scan[w] = nv; s_scan[4 + w] = nh; }
    __syncthreads();
    if (tid == 0) {
        tab_valid[t] = s_scan[0] + s_scan[1] + s_scan[2] + s_scan[3];
        tab_heads[t] = s_scan[4] + s_scan[5] + s_scan[6] + s_scan[7];
    }
    if (!want_runs) return;
    // The runs, for an update that goes by position (k_small_update): the ordered piece is still in LDS.  A run's row is
    // found where remap found its first pair's lookup: in the cache, or (a miss) in that lookup's row of the staging area
    // when the batch's missed rows are there, else in host memory.
    const SmallRunArgs& Q = S.run;
    // A run's length is the distance to the next run's first position: each thread looks at `per` consecutive positions,
    // a scan across the threads numbers the runs, their first positions are listed in LDS (in place of the values, which
    // are in vout by now), and each run reads its successor's.
    const uint32_t nv_all = s_scan[0] + s_scan[1] + s_scan[2] + s_scan[3];
    __syncthreads();                                   // (the scan below reuses s_scan)
    uint32_t* const s_first = s_val;
    const int per = (n + kBlock - 1) / kBlock;         // <= R
    const int q0 = tid * per;
    uint32_t heads = 0, cnt = 0;                       // bit i: position q0 + i starts a run
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const int q = q0 + i;
        if (i < per && q < n) {
            const uint32_t k = s_key[q];
            if (k != 0xFFFFFFFFu && (q == 0 || s_key[q - 1] != k)) { heads |= 1u << i; ++cnt; }
        }
    }
    uint32_t total;
    const uint32_t first_run = block_exclusive_scan(cnt, s_scan, &total);
    {
        uint32_t u = first_run;
#pragma unroll
        for (int i = 0; i < R; ++i)
            if (heads & (1u << i)) s_first[u++] = (uint32_t)(q0 + i);
    }
    __syncthreads();
    {
        uint32_t u = first_run;
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const int q = q0 + i;
            if (i >= per || q >= n) continue;
            int32_t len = 0, src = -1;
            if (heads & (1u << i)) {
                const uint32_t next = u + 1 < total ? s_first[u + 1] : nv_all;
                ++u;
                len = (int32_t)next - q;
                const int32_t l = s_loc[q];
                src = (l >= 0 && (l < Q.k || Q.staged)) ? l : -1;
            }
            Q.run_len[a + q] = len;
            Q.run_src[a + q] = src;
        }
    }
    // positions of this table that the sort did not take (more lookups than the caller stated) hold no run
    const int32_t b_all = min(max(off[(int64_t)(t + 1) * B], a), L);
    for (int32_t q = a + n + tid; q < b_all; q += kBlock) Q.run_len[q] = 0;
}

// Rows of the pinned host tables -> a staging area in HBM, `lpr` lanes per row (lane gl holds 16-byte piece gl of the
// `chunks` pieces of a row), kStageUnroll rows in flight per lane group.  list[0 .. min(*d_count, cap_rows)) names the
// rows (global row ids); row j goes to staging row j.  `flags` (may be null: every row): only rows whose flag equals
// `want` are copied.  `block` of `nblocks` workgroups share the job; s_rbase is LDS [num_tables + 1], filled here.
constexpr int kStageUnroll = 4;
struct StageArgs {
    const int32_t* list;
    const int32_t* d_count;
    u32x4* staging;
    int chunks, lpr;
    int64_t cap_rows;
    const uint8_t* flags;
    int want;
};
__device__ __forceinline__ void stage_rows_body(int block, int nblocks, const Meta* __restrict__ meta, int32_t* s_rbase,
                                                const StageArgs& S) {
    const int T = meta->num_tables;
    for (int t = threadIdx.x; t <= T; t += kBlock) s_rbase[t] = meta->row_base[t];
    __syncthreads();
    const int64_t n = min((int64_t)*S.d_count, S.cap_rows);
    const int gpb = kBlock / S.lpr;
    const int grp = threadIdx.x / S.lpr, gl = threadIdx.x % S.lpr;
    const int64_t stride = (int64_t)nblocks * gpb;
    const bool lane_on = gl < S.chunks;      // lpr >= chunks: one 16-byte piece per lane
    if (!lane_on || n <= 0) return;
    for (int64_t j0 = (int64_t)block * gpb + grp; j0 < n; j0 += stride * kStageUnroll) {
        // row numbers are clamped instead of guarded so that the id loads, then the row loads over the link,
        // are all issued back to back; only rows below n are written
        int32_t gid[kStageUnroll];
        bool need[kStageUnroll];
        u32x4 v[kStageUnroll];
#pragma unroll
        for (int u = 0; u < kStageUnroll; ++u) {
            const int64_t j = min(j0 + u * stride, n - 1);
            gid[u] = S.list[j];
            need[u] = !S.flags || S.flags[j] == S.want;
        }
#pragma unroll
        for (int u = 0; u < kStageUnroll; ++u) {
            if (need[u]) {
                const int t = upper_table(s_rbase, T, gid[u]);
                v[u] = __builtin_nontemporal_load((const u32x4*)meta->table[t] + (int64_t)(gid[u] - s_rbase[t]) * S.chunks + gl);
            }
        }
#pragma unroll
        for (int u = 0; u < kStageUnroll; ++u)
            if (need[u] && j0 + u * stride < n) S.staging[(j0 + u * stride) * S.chunks + gl] = v[u];
    }
}

__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// fp32 -> bf16, round to nearest even (NaN kept quiet)
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ uint32_t next_pow2_u32(uint32_t x) {
    return x <= 1 ? 1u : 1u << (32 - __builtin_clz(x - 1));
}

}  // namespace scars

namespace scars {
inline int next_pow2_host(int x) {
    int p = 1;
    while (p < x) p <<= 1;
    return p;
}
// how far the bag id is shifted up in a pair's value: the bits left over hold the lookup's place inside its bag
inline int bag_shift_host(int64_t G) {
    int bits = 1;
    while (bits < 31 && ((int64_t)1 << bits) < G) ++bits;
    return 32 - bits;
}
// lanes that walk one bag in bag_pairs: about the mean bag length, a power of two up to a wave
inline int pairs_lanes_per_bag(int64_t L, int64_t G) {
    const int64_t mean = L / (G > 1 ? G : 1);
    return next_pow2_host((int)(mean < 1 ? 1 : (mean > 64 ? 64 : mean)));
}
}  // namespace scars
