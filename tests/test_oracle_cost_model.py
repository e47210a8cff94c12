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
