/* CPU oracle for the skew-aware cached embedding-bag step -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, host-memory, synchronous statement of what each step of the hot path
 * computes, written from the paper's description (Section III: a ranked skew table over all
 * embeddings, the top entries kept on the device; Section II-B: a cached set C that removes
 * communication but changes no value; Section II / Fig. 1: per-sample lookups in tables that
 * live in main memory) and the plain definitions of a pooled sum and of an aggregated
 * gradient step.  Floating point is accumulated in fp64 and rounded once.
 *
 * Nothing here is shared with the HIP library: no header, no helper, no constant.  Only the
 * tests, the smoke check and the benchmark's cpu_baseline leg may load this library; the
 * product path never does.
 *
 * Conventions: T tables with rows[t] rows each, global row id gid = row_base[t] + idx with
 * row_base the exclusive prefix sum of rows; a batch is table-major CSR: offsets has T*B+1
 * entries, bag g = t*B + b owns lookups [offsets[g], offsets[g+1]) and indices are
 * table-local.  dtype 0 = fp32 rows, 1 = bf16 rows (uint16 storage).
 *
 * Every function returns 0, or ORA_ERR_INVALID_ARG / ORA_ERR_OFFSETS (nothing written), or
 * ORA_ERR_INDEX_RANGE (outputs written as if each out-of-range lookup were absent).
 */
#ifndef SCARS_ORACLE_H
#define SCARS_ORACLE_H
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ORA_OK 0
#define ORA_ERR_INVALID_ARG (-1)
#define ORA_ERR_INDEX_RANGE (-5)
#define ORA_ERR_OFFSETS (-6)

/* worker threads for the loops over independent outputs (bags, unique rows); returns the count in use */
int32_t ora_set_threads(int32_t n);

/* Section IV fixes the cache by a byte budget (128 MB .. 1024 MB): k = min(N, floor(budget / row_bytes)). */
int64_t ora_budget_rows(int64_t n_rows, int64_t row_bytes, int64_t budget_bytes);

/* Skew table (Section III): counts[gid] += 1 for every lookup of the stream, duplicates included. */
int32_t ora_histogram(int32_t T, const int64_t* rows, const int32_t* indices, const int32_t* offsets,
                      int64_t L, int64_t B, uint32_t* counts /* [N], accumulated into */);

/* Ranked skew table -> top k (Section III): order all rows by count descending, lower gid first
 * among equal counts; hot_gid[s] is the s-th row of that order, slot_of[gid] = s or -1. */
int32_t ora_hot_set(int64_t N, const uint32_t* counts, int64_t k, int32_t* hot_gid /* [k] */,
                    int32_t* slot_of /* [N] */);

/* Lookup into the cached layer (Section II-B, Section IV): slot[i] = slot_of[gid_i]; positions of
 * hits and of misses in ascending order; miss_gid[j] = gid of miss_pos[j]; n_out = {n_hit, n_miss}. */
int32_t ora_remap(int32_t T, const int64_t* rows, const int32_t* indices, const int32_t* offsets,
                  int64_t L, int64_t B, const int32_t* slot_of, int32_t* slot /* [L] */,
                  int32_t* hit_pos, int32_t* miss_pos, int32_t* miss_gid, int64_t* n_out /* [2] */);

/* Pooled sum (Fig. 1 step 2 with sum pooling): out[g][:] = sum of the bag's rows read straight from
 * the tables in main memory; no cache is involved. out is fp32 [T*B][D]. */
int32_t ora_embedding_bag_fwd(int32_t T, const int64_t* rows, int32_t D, int32_t dtype,
                              const void* const* tables, const int32_t* indices, const int32_t* offsets,
                              int64_t L, int64_t B, float* out);

/* Same sum, but a row whose slot_of is >= 0 is read from cache[slot] instead of its table
 * (Section II-B: a cached row replaces the transfer, never the value). */
int32_t ora_embedding_bag_fwd_cached(int32_t T, const int64_t* rows, int32_t D, int32_t dtype,
                                     const void* const* tables, const int32_t* slot_of, const void* cache,
                                     const int32_t* indices, const int32_t* offsets, int64_t L, int64_t B,
                                     float* out);

/* Coalescing (Section II-A, eq. (1)-(3)): instead of one embedding per lookup, send the list of UNIQUE missed
 * embeddings of the batch plus, per lookup, an index into that list.  unique_gid = the distinct values of
 * miss_gid in ascending order, inverse[j] = position of miss_gid[j] in it, *U = their number. */
int32_t ora_coalesce(int64_t n_miss, const int32_t* miss_gid, int32_t* unique_gid /* [n_miss] */,
                     int32_t* inverse /* [n_miss] */, int64_t* U);

/* Hot / normal samples (Section III): a sample is hot when every one of its lookups, over all T tables, falls
 * in the cached set (a sample without lookups is hot); is_hot[b] = 1/0, hot_ids / normal_ids list the sample
 * ids of each class in ascending order, n_out = {n_hot, n_normal}. */
int32_t ora_classify_samples(int32_t T, const int64_t* rows, const int32_t* indices, const int32_t* offsets,
                             int64_t L, int64_t B, const int32_t* slot_of, int32_t* is_hot /* [B] */,
                             int32_t* hot_ids /* [B] */, int32_t* normal_ids /* [B] */, int64_t* n_out /* [2] */);

/* Section III, separate mini-batches of hot and normal samples: the sub-batch of samples ids[0..n) (ascending),
 * table-major with n samples per table, lookups in their original order.  sub_offsets has T*n + 1 entries. */
int32_t ora_partition_batch(int32_t T, const int32_t* indices, const int32_t* offsets, int64_t L, int64_t B,
                            const int32_t* ids, int64_t n, int32_t* sub_indices, int32_t* sub_offsets, int64_t* L_sub);

/* Use of the cache by portion (the measurement behind Fig. 4 of Section IV: how many samples of a mini-batch
 * touch each successive portion of the hotness-ordered cache).  Portion p holds slots
 * [p * portion_rows, (p+1) * portion_rows); usage[p] = number of samples with at least one lookup whose slot
 * falls in portion p (slots at or beyond n_portions * portion_rows are not counted). */
int32_t ora_portion_usage(int32_t T, const int64_t* rows, const int32_t* indices, const int32_t* offsets,
                          int64_t L, int64_t B, const int32_t* slot_of, int64_t portion_rows, int32_t n_portions,
                          int32_t* usage /* [n_portions] */);

/* Expected communication per epoch with a cached set (Section II-B, eq. (6) with the batch size of eq. (7)).
 * P(e) = min(1, counts[e] / n_samples) (eq. (1)'s probability that a random sample refers to e, estimated from
 * the skew table); C = the first k rows in the order (count descending, lower id first);
 * b = (M - k*d) / a (eq. (7), real-valued; the call fails with ORA_ERR_INVALID_ARG if b < 1);
 *   cost = T*Q + (Q / b) * d * sum_{e not in C} (1 - (1 - P(e))^b)        (eq. (6), summed over the T features;
 * the first term is the indices, the second the embeddings, both in parameters).  *b_out receives b. */
int32_t ora_epoch_cost(int32_t T, int64_t N, const uint32_t* counts, int64_t n_samples, int64_t k, double M, double a,
                       double d, double Q, double* cost, double* b_out);

/* Brute force over every feasible k in [0, k_max]: the k with the smallest ora_epoch_cost (lowest k on ties). */
/* Eq. (8)-(12): the test for caching one more embedding.  C = first k rows of the ranking, e' the next one;
 * *lhs = 1 - (1 - P(e'))^b, *t1 as in eq. (12) with b' = b - d / a.  Communication per epoch falls iff lhs >= t1. */
int32_t ora_caching_gain(int64_t N, const uint32_t* counts, int64_t n_samples, int64_t k, double M, double a, double d,
                         double* lhs, double* t1);

int32_t ora_plan_brute(int32_t T, int64_t N, const uint32_t* counts, int64_t n_samples, int64_t k_max, double M, double a,
                       double d, double Q, int64_t* best_k, double* best_cost);

/* Lookups ordered by (gid, position): sorted_gid, sorted_bag (bag of each lookup), seg_start[r] = first
 * sorted position of the r-th distinct gid (seg_start[U] = number of valid lookups), unique_gid ascending. */
int32_t ora_bwd_segments(int32_t T, const int64_t* rows, const int32_t* indices, const int32_t* offsets,
                         int64_t L, int64_t B, int32_t* sorted_gid /* [L] */, int32_t* sorted_bag /* [L] */,
                         int32_t* seg_start /* [L+1] */, int32_t* unique_gid /* [L] */, int64_t* U);

/* Aggregated gradient step on the embedding rows (the "backward" and "optimization" stages of
 * Section IV): dW[r] = sum over lookups of r of grad_out[bag], then
 *   optimizer 0 (SGD):     w -= lr * dW
 *   optimizer 1 (Adagrad): G += dW^2 ; w -= lr * dW / (sqrt(G) + eps)      (element-wise, fp32 state)
 * Only rows that are looked up change.  report = 0: tables (and state) are updated in place.
 * report = 1: nothing is mutated; for the r-th unique gid (ascending) the fp64 values before the final
 * rounding go to new_rows[r][:], new_state[r][:] and the summed gradient to grad_rows[r][:]
 * (each [U][D] fp64, any may be NULL). */
int32_t ora_embedding_bag_bwd_update(int32_t T, const int64_t* rows, int32_t D, int32_t dtype,
                                     void* const* tables, float* const* state, int32_t optimizer,
                                     const int32_t* indices, const int32_t* offsets, int64_t L, int64_t B,
                                     const float* grad_out, float lr, float eps, int32_t report,
                                     double* new_rows, double* new_state, double* grad_rows);

#ifdef __cplusplus
}
#endif
#endif
