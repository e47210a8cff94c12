/* CPU oracle -- TEST INFRASTRUCTURE ONLY (see scars_oracle.h).  Plain C, fp64 accumulation,
 * one loop nest per definition; OpenMP only over independent outputs. */
#include "scars_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int g_threads = 1;

int32_t ora_set_threads(int32_t n) {
    if (n < 1) n = 1;
#ifdef _OPENMP
    g_threads = n;
#else
    g_threads = 1;
#endif
    return g_threads;
}

int64_t ora_budget_rows(int64_t n_rows, int64_t row_bytes, int64_t budget_bytes) {
    if (row_bytes <= 0 || budget_bytes <= 0) return 0;
    int64_t k = budget_bytes / row_bytes;
    return k < n_rows ? k : n_rows;
}

/* ---- shared argument checks and the (table, gid) of a lookup ------------------------------- */
static int check_batch(int32_t T, const int64_t* rows, const int32_t* indices, const int32_t* offsets,
                       int64_t L, int64_t B) {
    if (T < 1 || !rows || !offsets || L < 0 || B < 0 || (L > 0 && !indices)) return ORA_ERR_INVALID_ARG;
    int64_t G = (int64_t)T * B;
    if (offsets[0] != 0 || offsets[G] != L) return ORA_ERR_OFFSETS;
    for (int64_t g = 0; g < G; ++g)
        if (offsets[g + 1] < offsets[g]) return ORA_ERR_OFFSETS;
    return ORA_OK;
}

static int64_t* make_row_base(int32_t T, const int64_t* rows) {
    int64_t* rb = (int64_t*)malloc(sizeof(int64_t) * (size_t)(T + 1));
    rb[0] = 0;
    for (int32_t t = 0; t < T; ++t) rb[t + 1] = rb[t] + rows[t];
    return rb;
}

static float bf16_to_f32(uint16_t h) {
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* round-to-nearest-even of an fp32 value to bf16 */
static uint16_t f32_to_bf16(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u); /* NaN stays NaN */
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    return (uint16_t)(u >> 16);
}

static double load_elem(const void* base, int32_t dtype, int64_t off) {
    if (dtype == 0) return (double)((const float*)base)[off];
    return (double)bf16_to_f32(((const uint16_t*)base)[off]);
}

/* ---- histogram -------------------------------------------------------------------------- */
int32_t ora_histogram(int32_t T, const int64_t* rows, const int32_t* indices, const int32_t* offsets,
                      int64_t L, int64_t B, uint32_t* counts) {
    int rc = check_batch(T, rows, indices, offsets, L, B);
    if (rc) return rc;
    if (!counts) return ORA_ERR_INVALID_ARG;
    int64_t* rb = make_row_base(T, rows);
    int bad = 0;
    for (int32_t t = 0; t < T; ++t)
        for (int64_t b = 0; b < B; ++b) {
            int64_t g = (int64_t)t * B + b;
            for (int64_t i = offsets[g]; i < offsets[g + 1]; ++i) {
                int64_t idx = indices[i];
                if (idx < 0 || idx >= rows[t]) { bad = 1; continue; }
                counts[rb[t] + idx] += 1u;
            }
        }
    free(rb);
    return bad ? ORA_ERR_INDEX_RANGE : ORA_OK;
}

/* ---- hot set ------------------------------------------------------------------------------ */
typedef struct { uint32_t count; int32_t gid; } rank_item;

static int cmp_rank(const void* a, const void* b) {
    const rank_item* x = (const rank_item*)a;
    const rank_item* y = (const rank_item*)b;
    if (x->count != y->count) return x->count > y->count ? -1 : 1; /* larger count first */
    if (x->gid != y->gid) return x->gid < y->gid ? -1 : 1;         /* then lower id      */
    return 0;
}

int32_t ora_hot_set(int64_t N, const uint32_t* counts, int64_t k, int32_t* hot_gid, int32_t* slot_of) {
    if (N < 1 || N >= ((int64_t)1 << 31) || !counts || !slot_of || k < 0 || k > N || (k > 0 && !hot_gid))
        return ORA_ERR_INVALID_ARG;
    rank_item* all = (rank_item*)malloc(sizeof(rank_item) * (size_t)N);
    for (int64_t g = 0; g < N; ++g) { all[g].count = counts[g]; all[g].gid = (int32_t)g; }
    qsort(all, (size_t)N, sizeof(rank_item), cmp_rank);
    for (int64_t g = 0; g < N; ++g) slot_of[g] = -1;
    for (int64_t s = 0; s < k; ++s) { hot_gid[s] = all[s].gid; slot_of[all[s].gid] = (int32_t)s; }
    free(all);
    return ORA_OK;
}

/* ---- remap ------------------------------------------------------------------------------- */
int32_t ora_remap(int32_t T, const int64_t* rows, const int32_t* indices, const int32_t* offsets,
                  int64_t L, int64_t B, const int32_t* slot_of, int32_t* slot, int32_t* hit_pos,
                  int32_t* miss_pos, int32_t* miss_gid, int64_t* n_out) {
    int rc = check_batch(T, rows, indices, offsets, L, B);
    if (rc) return rc;
    if (!slot_of || !n_out || (L > 0 && (!slot || !hit_pos || !miss_pos || !miss_gid)))
        return ORA_ERR_INVALID_ARG;
    int64_t* rb = make_row_base(T, rows);
    int64_t nh = 0, nm = 0;
    int bad = 0;
    for (int32_t t = 0; t < T; ++t)
        for (int64_t i = offsets[(int64_t)t * B]; i < offsets[(int64_t)(t + 1) * B]; ++i) {
            int64_t idx = indices[i];
            if (idx < 0 || idx >= rows[t]) { bad = 1; slot[i] = -1; continue; }
            int64_t gid = rb[t] + idx;
            int32_t s = slot_of[gid];
            slot[i] = s;
            if (s >= 0) {
                hit_pos[nh++] = (int32_t)i;
            } else {
                miss_pos[nm] = (int32_t)i;
                miss_gid[nm] = (int32_t)gid;
                ++nm;
            }
        }
    n_out[0] = nh;
    n_out[1] = nm;
    free(rb);
    return bad ? ORA_ERR_INDEX_RANGE : ORA_OK;
}

/* ---- coalescing: unique missed rows and the per-lookup index into them ------------------------- */
typedef struct { int32_t gid; int32_t j; } miss_item;

static int cmp_miss(const void* a, const void* b) {
    const miss_item* x = (const miss_item*)a;
    const miss_item* y = (const miss_item*)b;
    if (x->gid != y->gid) return x->gid < y->gid ? -1 : 1;
    if (x->j != y->j) return x->j < y->j ? -1 : 1;
    return 0;
}

int32_t ora_coalesce(int64_t n_miss, const int32_t* miss_gid, int32_t* unique_gid, int32_t* inverse, int64_t* U) {
    if (n_miss < 0 || !U || (n_miss > 0 && (!miss_gid || !unique_gid || !inverse))) return ORA_ERR_INVALID_ARG;
    miss_item* m = (miss_item*)malloc(sizeof(miss_item) * (size_t)(n_miss > 0 ? n_miss : 1));
    for (int64_t j = 0; j < n_miss; ++j) { m[j].gid = miss_gid[j]; m[j].j = (int32_t)j; }
    qsort(m, (size_t)n_miss, sizeof(miss_item), cmp_miss);
    int64_t u = 0;
    for (int64_t s = 0; s < n_miss; ++s) {
        if (s == 0 || m[s].gid != m[s - 1].gid) unique_gid[u++] = m[s].gid;
        inverse[m[s].j] = (int32_t)(u - 1);
    }
    *U = u;
    free(m);
    return ORA_OK;
}

/* ---- hot / normal samples ------------------------------------------------------------------------ */
int32_t ora_classify_samples(int32_t T, const int64_t* rows, const int32_t* indices, const int32_t* offsets,
                             int64_t L, int64_t B, const int32_t* slot_of, int32_t* is_hot, int32_t* hot_ids,
                             int32_t* normal_ids, int64_t* n_out) {
    int rc = check_batch(T, rows, indices, offsets, L, B);
    if (rc) return rc;
    if (!slot_of || !n_out || (B > 0 && (!is_hot || !hot_ids || !normal_ids))) return ORA_ERR_INVALID_ARG;
    int64_t* rb = make_row_base(T, rows);
    int64_t nh = 0, nn = 0;
    int bad = 0;
    for (int64_t b = 0; b < B; ++b) {
        int hot = 1;
        for (int32_t t = 0; t < T; ++t) {
            int64_t g = (int64_t)t * B + b;
            for (int64_t i = offsets[g]; i < offsets[g + 1]; ++i) {
                int64_t idx = indices[i];
                if (idx < 0 || idx >= rows[t]) { bad = 1; continue; }
                if (slot_of[rb[t] + idx] < 0) hot = 0;
            }
        }
        is_hot[b] = hot;
        if (hot) hot_ids[nh++] = (int32_t)b; else normal_ids[nn++] = (int32_t)b;
    }
    n_out[0] = nh;
    n_out[1] = nn;
    free(rb);
    return bad ? ORA_ERR_INDEX_RANGE : ORA_OK;
}

/* ---- sub-batch of selected samples ---------------------------------------------------------------
 * Section III: hot and normal samples are trained in separate mini-batches.  The sub-batch of the samples
 * ids[0..n) (ascending sample numbers) keeps the table-major layout with n samples per table: its bag
 * t*n + j is bag t*B + ids[j] of the batch, lookups in their original order. */
int32_t ora_partition_batch(int32_t T, const int32_t* indices, const int32_t* offsets, int64_t L, int64_t B,
                            const int32_t* ids, int64_t n, int32_t* sub_indices, int32_t* sub_offsets, int64_t* L_sub) {
    if (T < 1 || B < 0 || L < 0 || n < 0 || n > B || !offsets || !sub_offsets || !L_sub || (n > 0 && !ids) ||
        (L > 0 && (!indices || !sub_indices)))
        return ORA_ERR_INVALID_ARG;
    for (int64_t j = 0; j < n; ++j)
        if (ids[j] < 0 || ids[j] >= B || (j > 0 && ids[j] <= ids[j - 1])) return ORA_ERR_INVALID_ARG;
    int64_t pos = 0;
    sub_offsets[0] = 0;
    for (int32_t t = 0; t < T; ++t) {
        for (int64_t j = 0; j < n; ++j) {
            int64_t g = (int64_t)t * B + ids[j];
            if (offsets[g] < 0 || offsets[g + 1] < offsets[g] || offsets[g + 1] > L) return ORA_ERR_OFFSETS;
            for (int64_t i = offsets[g]; i < offsets[g + 1]; ++i) sub_indices[pos++] = indices[i];
            sub_offsets[(int64_t)t * n + j + 1] = (int32_t)pos;
        }
    }
    *L_sub = pos;
    return ORA_OK;
}

/* ---- cache use by portion ------------------------------------------------------------------------ */
int32_t ora_portion_usage(int32_t T, const int64_t* rows, const int32_t* indices, const int32_t* offsets,
                          int64_t L, int64_t B, const int32_t* slot_of, int64_t portion_rows, int32_t n_portions,
                          int32_t* usage) {
    int rc = check_batch(T, rows, indices, offsets, L, B);
    if (rc) return rc;
    if (!slot_of || portion_rows < 1 || n_portions < 1 || !usage) return ORA_ERR_INVALID_ARG;
    int64_t* rb = make_row_base(T, rows);
    char* seen = (char*)malloc((size_t)n_portions);
    int bad = 0;
    for (int32_t p = 0; p < n_portions; ++p) usage[p] = 0;
    for (int64_t b = 0; b < B; ++b) {
        memset(seen, 0, (size_t)n_portions);
        for (int32_t t = 0; t < T; ++t) {
            int64_t g = (int64_t)t * B + b;
            for (int64_t i = offsets[g]; i < offsets[g + 1]; ++i) {
                int64_t idx = indices[i];
                if (idx < 0 || idx >= rows[t]) { bad = 1; continue; }
                int64_t s = slot_of[rb[t] + idx];
                if (s >= 0 && s / portion_rows < n_portions) seen[s / portion_rows] = 1;
            }
        }
        for (int32_t p = 0; p < n_portions; ++p) usage[p] += seen[p];
    }
    free(seen);
    free(rb);
    return bad ? ORA_ERR_INDEX_RANGE : ORA_OK;
}

/* ---- expected communication per epoch (eq. (6), (7)) ---------------------------------------------- */
int32_t ora_epoch_cost(int32_t T, int64_t N, const uint32_t* counts, int64_t n_samples, int64_t k, double M, double a,
                       double d, double Q, double* cost, double* b_out) {
    if (T < 1 || N < 1 || !counts || n_samples < 1 || k < 0 || k > N || a <= 0.0 || d <= 0.0 || !cost)
        return ORA_ERR_INVALID_ARG;
    const double b = (M - (double)k * d) / a;
    if (!(b >= 1.0)) return ORA_ERR_INVALID_ARG;
    int32_t* hot = (int32_t*)malloc(sizeof(int32_t) * (size_t)(k > 0 ? k : 1));
    int32_t* slot_of = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
    int rc = ora_hot_set(N, counts, k, hot, slot_of);
    if (rc) { free(hot); free(slot_of); return rc; }
    double sum = 0.0;
    for (int64_t e = 0; e < N; ++e) {
        if (slot_of[e] >= 0) continue;                       /* cached: no transfer */
        double p = (double)counts[e] / (double)n_samples;
        if (p > 1.0) p = 1.0;
        sum += 1.0 - pow(1.0 - p, b);
    }
    *cost = (double)T * Q + (Q / b) * d * sum;
    if (b_out) *b_out = b;
    free(hot);
    free(slot_of);
    return ORA_OK;
}

int32_t ora_plan_brute(int32_t T, int64_t N, const uint32_t* counts, int64_t n_samples, int64_t k_max, double M, double a,
                       double d, double Q, int64_t* best_k, double* best_cost) {
    if (!best_k || !best_cost || k_max < 0 || k_max > N) return ORA_ERR_INVALID_ARG;
    int found = 0;
    for (int64_t k = 0; k <= k_max; ++k) {
        double c, b;
        if (ora_epoch_cost(T, N, counts, n_samples, k, M, a, d, Q, &c, &b) != ORA_OK) continue;
        if (!found || c < *best_cost) { *best_cost = c; *best_k = k; found = 1; }
    }
    return found ? ORA_OK : ORA_ERR_INVALID_ARG;
}

/* Caching one more embedding e' (eq. (8)-(12)): with C = the first k rows of the ranking, e' = the next one,
 * b = (M - k d) / a and b' = b - d / a, communication per epoch falls iff
 *     1 - (1 - P(e'))^b  >=  t1 = sum_{e not in C'} (b (1 - (1 - P(e))^b') - b' (1 - (1 - P(e))^b)) / b'. */
int32_t ora_caching_gain(int64_t N, const uint32_t* counts, int64_t n_samples, int64_t k, double M, double a, double d,
                         double* lhs, double* t1) {
    if (N < 1 || !counts || n_samples < 1 || k < 0 || k >= N || a <= 0.0 || d <= 0.0 || !lhs || !t1)
        return ORA_ERR_INVALID_ARG;
    const double b = (M - (double)k * d) / a, b2 = b - d / a;
    if (!(b2 >= 1.0)) return ORA_ERR_INVALID_ARG;
    int32_t* hot = (int32_t*)malloc(sizeof(int32_t) * (size_t)(k + 1));
    int32_t* slot_of = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
    int rc = ora_hot_set(N, counts, k + 1, hot, slot_of);          /* C' = first k + 1 rows; e' = the last of them */
    if (rc) { free(hot); free(slot_of); return rc; }
    double pe = (double)counts[hot[k]] / (double)n_samples;
    if (pe > 1.0) pe = 1.0;
    *lhs = 1.0 - pow(1.0 - pe, b);
    double sum = 0.0;
    for (int64_t e = 0; e < N; ++e) {
        if (slot_of[e] >= 0) continue;
        double p = (double)counts[e] / (double)n_samples;
        if (p > 1.0) p = 1.0;
        sum += (b * (1.0 - pow(1.0 - p, b2)) - b2 * (1.0 - pow(1.0 - p, b))) / b2;
    }
    *t1 = sum;
    free(hot);
    free(slot_of);
    return ORA_OK;
}

/* ---- forward ----------------------------------------------------------------------------- */
static int32_t fwd_impl(int32_t T, const int64_t* rows, int32_t D, int32_t dtype, const void* const* tables,
                        const int32_t* slot_of, const void* cache, const int32_t* indices,
                        const int32_t* offsets, int64_t L, int64_t B, float* out) {
    int rc = check_batch(T, rows, indices, offsets, L, B);
    if (rc) return rc;
    if (D < 1 || (dtype != 0 && dtype != 1) || !tables || !out) return ORA_ERR_INVALID_ARG;
    int64_t* rb = make_row_base(T, rows);
    int64_t G = (int64_t)T * B;
    int bad = 0;
#pragma omp parallel for schedule(static) num_threads(g_threads) reduction(| : bad)
    for (int64_t g = 0; g < G; ++g) {
        int32_t t = (int32_t)(g / B);
        double* acc = (double*)calloc((size_t)D, sizeof(double));
        for (int64_t i = offsets[g]; i < offsets[g + 1]; ++i) {
            int64_t idx = indices[i];
            if (idx < 0 || idx >= rows[t]) { bad |= 1; continue; }
            const void* base = tables[t];
            int64_t row = idx;
            if (slot_of && slot_of[rb[t] + idx] >= 0) { base = cache; row = slot_of[rb[t] + idx]; }
            for (int32_t c = 0; c < D; ++c) acc[c] += load_elem(base, dtype, row * D + c);
        }
        for (int32_t c = 0; c < D; ++c) out[g * D + c] = (float)acc[c];
        free(acc);
    }
    free(rb);
    return bad ? ORA_ERR_INDEX_RANGE : ORA_OK;
}

int32_t ora_embedding_bag_fwd(int32_t T, const int64_t* rows, int32_t D, int32_t dtype,
                              const void* const* tables, const int32_t* indices, const int32_t* offsets,
                              int64_t L, int64_t B, float* out) {
    return fwd_impl(T, rows, D, dtype, tables, NULL, NULL, indices, offsets, L, B, out);
}

int32_t ora_embedding_bag_fwd_cached(int32_t T, const int64_t* rows, int32_t D, int32_t dtype,
                                     const void* const* tables, const int32_t* slot_of, const void* cache,
                                     const int32_t* indices, const int32_t* offsets, int64_t L, int64_t B,
                                     float* out) {
    if (!slot_of || !cache) return ORA_ERR_INVALID_ARG;
    return fwd_impl(T, rows, D, dtype, tables, slot_of, cache, indices, offsets, L, B, out);
}

/* ---- backward: ordering of lookups by (gid, position) ------------------------------------- */
typedef struct { int32_t gid; int32_t pos; int32_t bag; } pair_item;

static int cmp_pair(const void* a, const void* b) {
    const pair_item* x = (const pair_item*)a;
    const pair_item* y = (const pair_item*)b;
    if (x->gid != y->gid) return x->gid < y->gid ? -1 : 1;
    if (x->pos != y->pos) return x->pos < y->pos ? -1 : 1;
    return 0;
}

/* valid lookups as (gid, position, bag), sorted; returns their number, sets *bad on a range error */
static int64_t sorted_pairs(int32_t T, const int64_t* rows, const int32_t* indices, const int32_t* offsets,
                            int64_t L, int64_t B, pair_item** out, int* bad) {
    int64_t* rb = make_row_base(T, rows);
    pair_item* p = (pair_item*)malloc(sizeof(pair_item) * (size_t)(L > 0 ? L : 1));
    int64_t n = 0;
    for (int32_t t = 0; t < T; ++t)
        for (int64_t b = 0; b < B; ++b) {
            int64_t g = (int64_t)t * B + b;
            for (int64_t i = offsets[g]; i < offsets[g + 1]; ++i) {
                int64_t idx = indices[i];
                if (idx < 0 || idx >= rows[t]) { *bad = 1; continue; }
                p[n].gid = (int32_t)(rb[t] + idx);
                p[n].pos = (int32_t)i;
                p[n].bag = (int32_t)g;
                ++n;
            }
        }
    qsort(p, (size_t)n, sizeof(pair_item), cmp_pair);
    free(rb);
    *out = p;
    return n;
}

int32_t ora_bwd_segments(int32_t T, const int64_t* rows, const int32_t* indices, const int32_t* offsets,
                         int64_t L, int64_t B, int32_t* sorted_gid, int32_t* sorted_bag, int32_t* seg_start,
                         int32_t* unique_gid, int64_t* U) {
    int rc = check_batch(T, rows, indices, offsets, L, B);
    if (rc) return rc;
    if (!seg_start || !U || (L > 0 && (!sorted_gid || !sorted_bag || !unique_gid))) return ORA_ERR_INVALID_ARG;
    int bad = 0;
    pair_item* p;
    int64_t n = sorted_pairs(T, rows, indices, offsets, L, B, &p, &bad);
    int64_t u = 0;
    for (int64_t j = 0; j < n; ++j) {
        sorted_gid[j] = p[j].gid;
        sorted_bag[j] = p[j].bag;
        if (j == 0 || p[j].gid != p[j - 1].gid) {
            seg_start[u] = (int32_t)j;
            unique_gid[u] = p[j].gid;
            ++u;
        }
    }
    seg_start[u] = (int32_t)n;
    *U = u;
    free(p);
    return bad ? ORA_ERR_INDEX_RANGE : ORA_OK;
}

/* ---- backward: aggregated gradient and row update ----------------------------------------- */
int32_t ora_embedding_bag_bwd_update(int32_t T, const int64_t* rows, int32_t D, int32_t dtype,
                                     void* const* tables, float* const* state, int32_t optimizer,
                                     const int32_t* indices, const int32_t* offsets, int64_t L, int64_t B,
                                     const float* grad_out, float lr, float eps, int32_t report,
                                     double* new_rows, double* new_state, double* grad_rows) {
    int rc = check_batch(T, rows, indices, offsets, L, B);
    if (rc) return rc;
    if (D < 1 || (dtype != 0 && dtype != 1) || !tables || !grad_out || (optimizer != 0 && optimizer != 1) ||
        (optimizer == 1 && !state))
        return ORA_ERR_INVALID_ARG;
    int bad = 0;
    pair_item* p;
    int64_t n = sorted_pairs(T, rows, indices, offsets, L, B, &p, &bad);
    /* segment boundaries */
    int64_t* start = (int64_t*)malloc(sizeof(int64_t) * (size_t)(n + 1));
    int64_t u = 0;
    for (int64_t j = 0; j < n; ++j)
        if (j == 0 || p[j].gid != p[j - 1].gid) start[u++] = j;
    start[u] = n;
    int64_t* rb = make_row_base(T, rows);
    const double dlr = (double)lr, deps = (double)eps;
#pragma omp parallel for schedule(dynamic, 64) num_threads(g_threads)
    for (int64_t r = 0; r < u; ++r) {
        int64_t gid = p[start[r]].gid;
        int32_t t = 0;
        while (gid >= rb[t + 1]) ++t;
        int64_t row = gid - rb[t];
        double* dw = (double*)calloc((size_t)D, sizeof(double));
        for (int64_t j = start[r]; j < start[r + 1]; ++j) {
            const float* go = grad_out + (int64_t)p[j].bag * D;
            for (int32_t c = 0; c < D; ++c) dw[c] += (double)go[c];
        }
        for (int32_t c = 0; c < D; ++c) {
            double w = load_elem(tables[t], dtype, row * D + c);
            double acc = 0.0, wn;
            if (optimizer == 0) {
                wn = w - dlr * dw[c];
            } else {
                acc = (double)state[t][row * D + c] + dw[c] * dw[c];
                wn = w - dlr * dw[c] / (sqrt(acc) + deps);
            }
            if (report) {
                if (new_rows) new_rows[r * D + c] = wn;
                if (new_state && optimizer == 1) new_state[r * D + c] = acc;
                if (grad_rows) grad_rows[r * D + c] = dw[c];
            } else {
                if (dtype == 0) ((float*)tables[t])[row * D + c] = (float)wn;
                else ((uint16_t*)tables[t])[row * D + c] = f32_to_bf16((float)wn);
                if (optimizer == 1) state[t][row * D + c] = (float)acc;
            }
        }
        free(dw);
    }
    free(rb);
    free(start);
    free(p);
    return bad ? ORA_ERR_INDEX_RANGE : ORA_OK;
}
