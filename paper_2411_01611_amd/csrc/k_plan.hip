// Budget chooser: the expected-communication model of the paper's Section II-B evaluated on the skew table.
//
// eq. (6): with the set C cached, an epoch of Q samples in batches of b communicates, per feature,
//   Q + (Q / b) * d * sum_{e not in C} (1 - (1 - P(e))^b)      (indices + distinct uncached embeddings),
// and eq. (7) ties the batch size to the cache: b = (M - |C| d) / a.  P(e) depends on e only through its
// count, and C is a prefix of the ranking by count, so the sum needs only the "count of counts": how many rows
// have each count value.  One kernel builds that table (LDS bins for the many small counts, global bins up to
// 65535, a short list for the few larger ones); the search over |C| is host arithmetic on it.
#include <algorithm>
#include <cmath>

#include "scars_dev.h"

namespace scars {

constexpr int kCcLds = 2048;

__global__ __launch_bounds__(kBlock) void k_count_of_counts(const uint32_t* __restrict__ counts, int64_t N,
                                                            uint32_t* __restrict__ cc, uint32_t* __restrict__ big,
                                                            uint32_t* __restrict__ n_big) {
    __shared__ uint32_t s_h[kCcLds];
    for (int i = threadIdx.x; i < kCcLds; i += kBlock) s_h[i] = 0;
    __syncthreads();
    for (int64_t base = (int64_t)blockIdx.x * kBlock; base < N; base += (int64_t)gridDim.x * kBlock) {
        const int64_t g = base + threadIdx.x;
        const bool in = g < N;
        const uint32_t c = in ? counts[g] : 0u;
        // most rows of a wave share one small count: one LDS atomic for the wave then
        const uint64_t act = ballot64(in);
        if (act) {
            const int leader = __ffsll((unsigned long long)act) - 1;
            const uint32_t c0 = __shfl(c, leader, 64);
            const uint64_t same = ballot64(in && c == c0);
            if (same == act && c0 < kCcLds) {
                if (lane_id() == leader) atomicAdd(&s_h[c0], (uint32_t)__popcll(act));
            } else if (in) {
                if (c < kCcLds) atomicAdd(&s_h[c], 1u);
                else if (c < kPlanBins) atomicAdd(&cc[c], 1u);
                else {
                    const uint32_t j = atomicAdd(n_big, 1u);
                    if (j < kPlanBigCap) big[j] = c;
                }
            }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kCcLds; i += kBlock)
        if (s_h[i]) atomicAdd(&cc[i], s_h[i]);
}

hipError_t launch_count_of_counts(scars_handle* h, hipStream_t s) {
    Workspace& ws = h->ws;
    hipError_t e = launch_fill_u32(h, s, ws.plan_cc, kPlanBins + kPlanBigCap + 4, 0u);
    if (e != hipSuccess) return e;
    Timed t(h, s, "count_of_counts");
    const int grid = (int)std::min<int64_t>(div_up(h->N, kBlock), 256 * 16);
    hipLaunchKernelGGL(k_count_of_counts, dim3(grid), dim3(kBlock), 0, s, h->buf.counts, h->N, ws.plan_cc,
                       ws.plan_cc + kPlanBins, ws.plan_cc + kPlanBins + kPlanBigCap);
    return hipGetLastError();
}

// ---- host arithmetic -------------------------------------------------------------------------------------
// classes: (count, rows with that count), count descending
double plan_cost(const std::vector<std::pair<uint32_t, int64_t>>& classes, int T, int64_t n_samples, int64_t k, double M,
                 double a, double d, double Q, double* b_out) {
    const double b = (M - (double)k * d) / a;
    if (b_out) *b_out = b;
    if (!(b >= 1.0)) return INFINITY;
    double sum = 0.0;
    int64_t before = 0;                                   // rows in hotter classes
    for (const auto& cl : classes) {
        const int64_t cached = std::min<int64_t>(std::max<int64_t>(k - before, 0), cl.second);
        before += cl.second;
        const int64_t rest = cl.second - cached;
        if (rest == 0 || cl.first == 0) continue;         // count 0: P = 0, contributes nothing
        const double p = std::min(1.0, (double)cl.first / (double)n_samples);
        sum += (double)rest * (1.0 - std::pow(1.0 - p, b));
    }
    return (double)T * Q + (Q / b) * d * sum;
}

}  // namespace scars
