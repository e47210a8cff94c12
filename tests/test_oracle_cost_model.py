"""Pins for the oracle's expected-communication model (paper Section II-A/II-B, eq. (2)-(7))."""
import math

import numpy as np

from paper_2411_01611_amd import synth


def test_cost_uniform_closed_form(ora):
    # uniform P(e) = 1/n over n rows, k cached: sum = (n - k) * (1 - (1 - 1/n)^b), eq. (6) by hand
    n, S = 200, 200 * 50                                   # every row counted 50 times in 10000 samples: P = 1/200
    counts = np.full(n, 50, dtype=np.uint32)
    M, a, d, Q, T = 1.0e6, 1000.0, 16.0, 1.0e5, 1
    for k in (0, 1, 57, 200):
        rc, cost, b = ora.epoch_cost(T, counts, S, k, M, a, d, Q)
        assert rc == 0
        b_ref = (M - k * d) / a                            # eq. (7)
        assert abs(b - b_ref) < 1e-9
        ref = T * Q + (Q / b_ref) * d * (n - k) * (1.0 - (1.0 - 1.0 / n) ** b_ref)
        assert abs(cost - ref) <= 1e-12 * ref


def test_cost_reduces_to_batch_communication_without_overlap(ora):
    # b = 1 (M = a, nothing cached): 1 - (1 - P)^1 = P, the embeddings term is Q * d * sum P = Q * d: eq. (4)'s
    # "communicating the batch" plus the indices of eq. (5)
    wl = synth.workload("tiny")
    s = synth.Sampler(wl)
    idx, off = s.batch(0, True)
    rc, counts = ora.histogram(wl.rows, idx.numpy(), off.numpy(), wl.batch)
    T, S = wl.num_tables, wl.batch
    rc, cost, b = ora.epoch_cost(T, counts, S, 0, 500.0, 500.0, 16.0, 1000.0)
    assert rc == 0 and b == 1.0
    assert abs(cost - (T * 1000.0 + 1000.0 * 16.0 * T)) < 1e-6       # sum of P over each of the T features is 1


def test_expected_unique_is_the_embedding_term(ora):
    # eq. (2): sum_e 1 - (1 - P(e))^b is the expected number of distinct rows in a batch of b; check the oracle's
    # sum (through its cost) against the number of distinct rows actually drawn
    wl = synth.workload("tiny", batch=2048)
    s = synth.Sampler(wl)
    T = wl.num_tables
    # exact probabilities as "counts" over a large virtual sample
    S = 10 ** 8
    counts = np.concatenate([np.round(s.row_probs(t).numpy() * S) for t in range(T)]).astype(np.uint32)
    b = 2048.0
    rc, cost, bb = ora.epoch_cost(T, counts, S, 0, b * 10.0, 10.0, 1.0, b)     # Q = b: one batch; d = 1
    EU = cost - T * b                                                           # (Q/b) * d * sum = sum
    idx, off = s.batch(0)
    U = sum(np.unique(idx[int(off[t * wl.batch]):int(off[(t + 1) * wl.batch])].numpy()).size for t in range(T))
    assert abs(U - EU) < 5 * math.sqrt(EU)


def test_caching_lowers_cost_at_fixed_batch_and_tradeoff_exists(ora):
    wl = synth.workload("tiny")
    s = synth.Sampler(wl)
    counts = None
    for p in range(16):
        idx, off = s.batch(p, True)
        rc, counts = ora.histogram(wl.rows, idx.numpy(), off.numpy(), wl.batch, counts)
    S, T, d, Q = 16 * wl.batch, wl.num_tables, 16.0, 1.0e6
    # a huge M keeps b almost constant: cost must fall monotonically with k
    prev = None
    for k in (0, 10, 100, 1000, 10000):
        rc, cost, b = ora.epoch_cost(T, counts, S, k, 1.0e12, 1.0e9, d, Q)
        assert rc == 0 and (prev is None or cost <= prev)
        prev = cost
    # a tight M: caching everything leaves no room for a batch (b < 1 is refused) and the optimum is interior
    M, a = 40000 * d * 0.6, 2000.0
    assert ora.epoch_cost(T, counts, S, 40000, M, a, d, Q)[0] != 0
    rc, bk, bc = ora.plan_brute(T, counts[:2000], S, 1500, 2000 * d * 0.6, 200.0, d, Q)
    assert rc == 0 and 0 < bk < 1500
    c0 = ora.epoch_cost(T, counts[:2000], S, 0, 2000 * d * 0.6, 200.0, d, Q)[1]
    assert bc < c0


def test_growth_with_five_times_rows_and_batch_stays_below_five(ora):
    # end of Section II-B: with 5x the embeddings and 5x the batch, sending each distinct embedding once grows the
    # per-batch communication by less than the 5x of sending every looked-up embedding; least for the light-tailed
    # rank distributions.  The paper does not give its parameters; these are ours: one feature, 2*10^5 -> 10^6 rows,
    # b = 2048 -> 10240, d = 64, Zipf exponent 1, exponential and half-normal with a scale of 2000 ranks (absolute,
    # so the added rows extend the tail).  Evaluated with the oracle's eq. (6) at k = 0 and Q = b (one batch).
    N0, b0, d, S = 200_000, 2048.0, 64.0, 10 ** 9
    j = lambda n: np.arange(n, dtype=np.float64)
    dists = {"zipf": lambda n: 1.0 / (j(n) + 1.0),
             "exp": lambda n: np.exp(-j(n) / 2000.0),
             "halfnormal": lambda n: np.exp(-(j(n) / 2000.0) ** 2 / 2.0)}
    growth = {}
    for name, w in dists.items():
        cost = []
        for n, b in ((N0, b0), (5 * N0, 5 * b0)):
            p = w(n)
            counts = np.round(p / p.sum() * S).astype(np.uint32)
            rc, c, bb = ora.epoch_cost(1, counts, S, 0, b * 1000.0, 1000.0, d, b)
            assert rc == 0 and abs(bb - b) < 1e-9
            cost.append(c)
        growth[name] = cost[1] / cost[0]
    assert growth["exp"] < growth["zipf"] < 5.0 and growth["halfnormal"] < growth["zipf"]
    assert growth["exp"] < 3.0 and growth["halfnormal"] < 3.0


def test_caching_one_more_row_criterion_agrees_with_the_cost_difference(ora):
    # eq. (11)/(12) is eq. (8) <= 0 rearranged: lhs >= t1 exactly when the epoch cost of eq. (6) does not rise from k
    # to k + 1 cached rows; and t1 against its definition written with numpy.  Two settings: a skewed table with
    # a > d (the regime in which the paper says caching generally helps: it does, at every k), and a flat table with
    # a < d, where giving up batch size for one more row does not pay until most rows are cached.
    wl = synth.workload("tiny")
    s = synth.Sampler(wl)
    skewed = None
    for p in range(8):
        idx, off = s.batch(p, True)
        rc, skewed = ora.histogram(wl.rows, idx.numpy(), off.numpy(), wl.batch, skewed)
    skewed = skewed[:3000]
    d, Q, T = 16.0, 1.0e6, 1
    outcomes = {}
    for name, counts, S, M, a, ks in (("skewed, a > d", skewed, 8 * wl.batch, 3000 * d * 0.6, 150.0, (0, 1, 5, 50, 200)),
                                      ("flat, a < d", np.ones(3000, dtype=np.uint32), 3000, 3000 * d * 0.5, 5.0,
                                       (0, 100, 500, 1000, 1400))):
        order = np.lexsort((np.arange(counts.size), -counts.astype(np.int64)))
        P = np.minimum(1.0, counts.astype(np.float64) / S)
        seen = []
        for k in ks:
            rc, lhs, t1 = ora.caching_gain(counts, S, k, M, a, d)
            assert rc == 0
            b = (M - k * d) / a
            b2 = b - d / a
            rest = P[order[k + 1:]]
            t1_ref = np.sum((b * (1 - (1 - rest) ** b2) - b2 * (1 - (1 - rest) ** b)) / b2)
            assert abs(lhs - (1 - (1 - P[order[k]]) ** b)) < 1e-14 and abs(t1 - t1_ref) <= 1e-9 * max(1.0, abs(t1_ref))
            c0 = ora.epoch_cost(T, counts, S, k, M, a, d, Q)[1]
            c1 = ora.epoch_cost(T, counts, S, k + 1, M, a, d, Q)[1]
            assert abs(c1 - c0) > 1e-9 * c0 and (lhs >= t1) == (c1 <= c0)
            seen.append(bool(lhs >= t1))
        outcomes[name] = seen
    assert outcomes["skewed, a > d"] == [True] * 5
    assert outcomes["flat, a < d"] == [False, False, False, True, True]
    # refused: nothing left to cache, or no room for a batch of one after caching one more
    assert ora.caching_gain(skewed, 8 * wl.batch, 3000, 1e6, 10.0, d)[0] != 0
    assert ora.caching_gain(skewed, 8 * wl.batch, 10, 10 * d + 20.0, 10.0, d)[0] != 0


def _cost_numpy(T, counts, S, k, M, a, d, Q):
    """Eq. (6) with eq. (7)'s batch size, restated with numpy: the first k rows by (count descending, row ascending)
    are cached; None when no batch of one sample fits."""
    b = (M - k * d) / a
    if not b >= 1.0:
        return None
    order = np.lexsort((np.arange(counts.size), -counts.astype(np.int64)))
    p = np.minimum(1.0, counts[order][k:].astype(np.float64) / S)
    return T * Q + (Q / b) * d * float(np.sum(1.0 - (1.0 - p) ** b))


def test_plan_brute_is_the_first_minimum_of_the_cost_over_every_feasible_k(ora):
    """ora_plan_brute against an argmin written with numpy over a numpy restatement of the cost: an interior optimum,
    an optimum at k_max (a > d: caching always pays), an optimum at the last feasible k before k_max (the rest leaves
    no room for a sample), and a tie (rows never seen add nothing: the smallest such k wins)."""
    rng = np.random.default_rng(11)
    T, d, Q = 3, 16.0, 1.0e5

    def check(counts, S, k_max, M, a):
        costs = [_cost_numpy(T, counts, S, k, M, a, d, Q) for k in range(k_max + 1)]
        feas = [(c, k) for k, c in enumerate(costs) if c is not None]
        want_c, want_k = min(feas, key=lambda ck: (ck[0], ck[1]))
        rc, bk, bc = ora.plan_brute(T, counts, S, k_max, M, a, d, Q)
        assert rc == 0
        # equal to rounding: the two sums add the same terms in different orders
        near = [k for c, k in feas if abs(c - want_c) <= 1e-9 * want_c]
        assert bk in near and abs(bc - want_c) <= 1e-9 * want_c
        return bk, want_k, len(feas)

    zipf = np.round(2000.0 / np.arange(1, 401) ** 1.1).astype(np.uint32)
    rng.shuffle(zipf)
    S = 4000
    # interior optimum: a tight device (M), cheap samples
    bk, wk, nf = check(zipf, S, 400, 400 * d * 0.6, 20.0)
    assert bk == wk and 0 < bk < 400 and nf < 401
    # a > d and plenty of room: every cached row lowers the cost, the optimum is k_max itself
    bk, wk, nf = check(zipf, S, 150, 1.0e7, 64.0)
    assert bk == wk == 150 and nf == 151
    # k_max beyond what leaves room for one sample: the optimum is the last feasible k, not k_max
    M = 100 * d + 64.0                                   # b(k) = (M - k d) / a >= 1  <=>  k <= 100
    bk, wk, nf = check(zipf, S, 150, M, 64.0)
    assert nf == 101 and bk == wk <= 100
    # a tie: beyond the 5 rows that were ever seen nothing is left to send, and with a = d * 1e9 the batch size does
    # not move: the cost is the same for every k >= 5 and the smallest of them is reported
    seen = np.zeros(60, dtype=np.uint32)
    seen[[3, 17, 18, 40, 59]] = [9, 2, 2, 7, 1]
    rc, bk, bc = ora.plan_brute(T, seen, 100, 60, 1.0e15, d * 1.0e9, d, Q)
    assert rc == 0 and bk == 5 and bc == T * Q
    # nothing feasible at all
    assert ora.plan_brute(T, seen, 100, 60, 10.0, 64.0, d, Q)[0] != 0
