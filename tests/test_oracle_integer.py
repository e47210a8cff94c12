"""Pins for the oracle's integer steps: histogram, hot set, remap, sorted segments.

Each pin is something other than the oracle itself: a numpy library routine used as a special case,
a brute-force loop, a closed form from the paper, or an invariant that any correct result satisfies.
"""
import math

import numpy as np

from paper_2411_01611_amd import synth
from util import bag_of, gids_of


def _batch(wl, bid=0, profile=False):
    idx, off = synth.Sampler(wl).batch(bid, profile)
    return idx.numpy(), off.numpy()


# ------------------------------------------------------------------ histogram
def test_histogram_matches_bincount_and_mass(ora):
    for name, kw in (("tiny", {}), ("multi_hot", {"scale": 0.01}), ("dlrm_onehot", {"scale": 0.002})):
        wl = synth.workload(name, **kw)
        idx, off = _batch(wl, 0, True)
        rc, counts = ora.histogram(wl.rows, idx, off, wl.batch)
        assert rc == 0 and counts.dtype == np.uint32
        ref = np.bincount(gids_of(wl, idx, off), minlength=wl.total_rows)
        assert np.array_equal(counts, ref)
        assert int(counts.sum()) == idx.shape[0]


def test_histogram_brute_force_and_accumulation(ora):
    wl = synth.workload("tiny")
    s = synth.Sampler(wl)
    total = np.zeros(wl.total_rows, dtype=np.int64)
    counts = None
    for p in range(3):
        idx, off = s.batch(p, True)
        idx, off = idx.numpy(), off.numpy()
        for t in range(wl.num_tables):
            for b in range(wl.batch):
                g = t * wl.batch + b
                for i in range(off[g], off[g + 1]):
                    total[wl.row_base[t] + idx[i]] += 1
        rc, counts = ora.histogram(wl.rows, idx, off, wl.batch, counts)
        assert rc == 0
    assert np.array_equal(counts.astype(np.int64), total)


def test_histogram_counts_duplicates_inside_a_bag(ora):
    rows = [5]
    off = np.array([0, 4], dtype=np.int32)
    idx = np.array([3, 3, 3, 1], dtype=np.int32)
    rc, c = ora.histogram(rows, idx, off, 1)
    assert rc == 0 and c.tolist() == [0, 1, 0, 3, 0]


# ------------------------------------------------------------------ hot set
def _lexsort_top(counts, k):
    order = np.lexsort((np.arange(counts.shape[0]), -counts.astype(np.int64)))
    return order[:k].astype(np.int32)


def test_hot_set_matches_lexsort(ora):
    wl = synth.workload("tiny")
    s = synth.Sampler(wl)
    counts = None
    for p in range(8):
        idx, off = s.batch(p, True)
        _, counts = ora.histogram(wl.rows, idx.numpy(), off.numpy(), wl.batch, counts)
    k = ora.budget_rows(wl.total_rows, wl.row_bytes, wl.budget_bytes)
    assert k == 4000
    rc, hot, slot_of = ora.hot_set(counts, k)
    assert rc == 0
    assert np.array_equal(hot, _lexsort_top(counts, k))
    # invariants: bijection, and the ordering rule across the boundary
    assert np.array_equal(slot_of[hot], np.arange(k))
    assert int((slot_of >= 0).sum()) == k
    cold = np.nonzero(slot_of < 0)[0]
    cmin = counts[hot].min()
    assert counts[cold].max() <= cmin
    tie_cold = cold[counts[cold] == cmin]
    tie_hot = hot[counts[hot] == cmin]
    if tie_cold.size and tie_hot.size:
        assert tie_hot.max() < tie_cold.min()
    # slot order is hotness order
    ch = counts[hot].astype(np.int64)
    assert np.all(np.diff(ch) <= 0)
    same = np.diff(ch) == 0
    assert np.all(np.diff(hot.astype(np.int64))[same] > 0)


def test_hot_set_tie_cases(ora):
    # all counts equal: the k lowest ids win
    rc, hot, slot_of = ora.hot_set(np.full(10, 7, dtype=np.uint32), 4)
    assert hot.tolist() == [0, 1, 2, 3] and slot_of.tolist() == [0, 1, 2, 3] + [-1] * 6
    # k = 0 and k = N
    rc, hot, slot_of = ora.hot_set(np.array([3, 1, 2], dtype=np.uint32), 0)
    assert rc == 0 and hot.size == 0 and slot_of.tolist() == [-1, -1, -1]
    rc, hot, slot_of = ora.hot_set(np.array([3, 1, 2, 3], dtype=np.uint32), 4)
    assert hot.tolist() == [0, 3, 2, 1] and slot_of.tolist() == [0, 3, 2, 1]
    # boundary inside a tie class that spans two tables (rows 0..2 | 3..5): counts 5,1,1 | 1,9,1 ; k = 4
    c = np.array([5, 1, 1, 1, 9, 1], dtype=np.uint32)
    rc, hot, slot_of = ora.hot_set(c, 4)
    assert hot.tolist() == [4, 0, 1, 2] and slot_of.tolist() == [1, 2, 3, -1, 0, -1]
    # zero-count rows are eligible as the last tie class
    rc, hot, _ = ora.hot_set(np.array([0, 0, 4, 0], dtype=np.uint32), 3)
    assert hot.tolist() == [2, 0, 1]
    # large counts compare as unsigned
    rc, hot, _ = ora.hot_set(np.array([1, 0xFFFFFFFF, 0x80000000], dtype=np.uint32), 2)
    assert hot.tolist() == [1, 2]


def test_budget_rows(ora):
    assert ora.budget_rows(100, 64, 0) == 0
    assert ora.budget_rows(100, 64, 63) == 0            # smaller than one row: nothing cached
    assert ora.budget_rows(100, 64, 64) == 1
    assert ora.budget_rows(100, 64, 64 * 100 + 5) == 100
    assert ora.budget_rows(100, 64, 10 ** 12) == 100
    assert ora.budget_rows(40_000_000, 512, 2_000_000_000) == 3_906_250


# ------------------------------------------------------------------ remap
def _build(ora, wl, nprofile=8):
    s = synth.Sampler(wl)
    counts = None
    for p in range(nprofile):
        idx, off = s.batch(p, True)
        _, counts = ora.histogram(wl.rows, idx.numpy(), off.numpy(), wl.batch, counts)
    k = ora.budget_rows(wl.total_rows, wl.row_bytes, wl.budget_bytes)
    _, hot, slot_of = ora.hot_set(counts, k)
    return s, counts, hot, slot_of


def test_remap_invariants(ora):
    for name, kw in (("tiny", {}), ("multi_hot", {"scale": 0.01})):
        wl = synth.workload(name, **kw)
        s, counts, hot, slot_of = _build(ora, wl)
        idx, off = s.batch(0)
        idx, off = idx.numpy(), off.numpy()
        L = idx.shape[0]
        rc, slot, hit, miss, mg = ora.remap(wl.rows, idx, off, wl.batch, slot_of)
        assert rc == 0
        gid = gids_of(wl, idx, off)
        assert np.array_equal(slot, slot_of[gid])                 # numpy gather as the special case
        assert hit.size + miss.size == L                           # every lookup is a hit or a miss
        assert np.all(np.diff(hit) > 0) and np.all(np.diff(miss) > 0)
        assert np.array_equal(np.sort(np.concatenate([hit, miss])), np.arange(L))
        assert np.all(slot[hit] >= 0) and np.all(slot[miss] == -1)
        assert np.array_equal(mg, gid[miss])
        assert np.array_equal(hot[slot[hit]], gid[hit])


def test_remap_no_cache_is_all_miss_and_full_cache_all_hit(ora):
    # eq. (4): without caching every lookup is communicated
    wl = synth.workload("tiny")
    idx, off = _batch(wl)
    none = np.full(wl.total_rows, -1, dtype=np.int32)
    rc, slot, hit, miss, mg = ora.remap(wl.rows, idx, off, wl.batch, none)
    assert hit.size == 0 and miss.size == idx.shape[0] and np.all(slot == -1)
    full = np.arange(wl.total_rows, dtype=np.int32)
    rc, slot, hit, miss, mg = ora.remap(wl.rows, idx, off, wl.batch, full)
    assert miss.size == 0 and hit.size == idx.shape[0]


def test_hit_rate_matches_cached_probability_mass(ora):
    # Section II-B / eq. (6): a cached set C removes exactly the lookups that fall in C, so the expected
    # hit rate is sum_{e in C} P(e).  Ideal hot set = top-k by true probability, per table.
    wl = synth.workload("tiny", batch=20_000)
    s = synth.Sampler(wl)
    slot_of = np.full(wl.total_rows, -1, dtype=np.int32)
    mass = 0.0
    nxt = 0
    for t in range(wl.num_tables):
        p = s.row_probs(t).numpy()
        top = np.argsort(-p, kind="stable")[:1000]
        slot_of[wl.row_base[t] + top] = np.arange(nxt, nxt + 1000)
        nxt += 1000
        mass += p[top].sum() / wl.num_tables
    idx, off = s.batch(0)
    rc, slot, hit, miss, mg = ora.remap(wl.rows, idx.numpy(), off.numpy(), wl.batch, slot_of)
    L = idx.numel()
    rate = hit.size / L
    assert abs(rate - mass) < 5 * math.sqrt(mass * (1 - mass) / L)
    assert 0.75 < mass < 0.9


# ------------------------------------------------------------------ sorted segments
def test_segments_properties_and_argsort(ora):
    for name, kw in (("tiny", {}), ("multi_hot", {"scale": 0.01})):
        wl = synth.workload(name, **kw)
        idx, off = _batch(wl)
        L = idx.shape[0]
        rc, sg, sb, ss, ug = ora.bwd_segments(wl.rows, idx, off, wl.batch)
        assert rc == 0 and sg.shape[0] == L
        gid = gids_of(wl, idx, off)
        order = np.argsort(gid, kind="stable")                    # library routine as the special case
        assert np.array_equal(sg, gid[order])
        assert np.array_equal(sb, bag_of(off, L)[order])
        uniq, first = np.unique(gid, return_index=False), None
        assert np.array_equal(ug, uniq)
        assert ss[0] == 0 and ss[-1] == L and np.all(np.diff(ss) > 0)
        assert np.array_equal(sg[ss[:-1]], ug)
        assert np.all(np.diff(sg) >= 0)


def test_unique_count_matches_expected_unique_formula(ora):
    # eq. (2): E[U] = sum_e 1 - (1 - P(e))^b per feature; Var[U] <= E[U] (negatively associated indicators)
    wl = synth.workload("tiny", batch=4096)
    s = synth.Sampler(wl)
    idx, off = s.batch(0)
    rc, sg, sb, ss, ug = ora.bwd_segments(wl.rows, idx.numpy(), off.numpy(), wl.batch)
    EU = 0.0
    for t in range(wl.num_tables):
        p = s.row_probs(t).numpy()
        EU += np.sum(1.0 - (1.0 - p) ** wl.batch)
    assert abs(ug.size - EU) < 5 * math.sqrt(EU)
    # uniform special case n * (1 - (1 - 1/n)^b)
    wl = synth.workload("tiny", batch=4096, zipf_s=None)
    idx, off = synth.Sampler(wl).batch(0)
    rc, sg, sb, ss, ug = ora.bwd_segments(wl.rows, idx.numpy(), off.numpy(), wl.batch)
    EU = 4 * 10_000 * (1 - (1 - 1e-4) ** 4096)
    assert abs(ug.size - EU) < 5 * math.sqrt(EU)


def test_expected_unique_golden_closed_form():
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "expected_unique_closed_form.txt")
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        n, b, want = line.split()
        n, b, want = int(n), int(b), float(want)
        p = np.full(n, 1.0 / n)
        assert abs(np.sum(1 - (1 - p) ** b) - want) < 1e-6


# ------------------------------------------------------------------ error behaviour
def test_errors(ora):
    rows = [4, 3]
    off = np.array([0, 1, 2, 3, 4], dtype=np.int32)
    idx = np.array([0, 3, 2, 1], dtype=np.int32)
    slot_of = np.array([0, -1, 1, -1, 2, -1, -1], dtype=np.int32)
    bad_off = np.array([0, 2, 1, 3, 4], dtype=np.int32)
    assert ora.histogram(rows, idx, bad_off, 2)[0] == ora.ERR_OFFSETS
    assert ora.remap(rows, idx, bad_off, 2, slot_of)[0] == ora.ERR_OFFSETS
    assert ora.histogram(rows, idx, np.array([0, 1, 2, 3, 5], dtype=np.int32), 2)[0] == ora.ERR_OFFSETS
    # an out-of-range index is reported and treated as absent
    bad_idx = np.array([0, 4, 3, 1], dtype=np.int32)          # 4 >= rows[0]; 3 >= rows[1]
    rc, c = ora.histogram(rows, bad_idx, off, 2)
    assert rc == ora.ERR_INDEX_RANGE and c.tolist() == [1, 0, 0, 0, 0, 1, 0]
    rc, slot, hit, miss, mg = ora.remap(rows, bad_idx, off, 2, slot_of)
    assert rc == ora.ERR_INDEX_RANGE and slot.tolist() == [0, -1, -1, -1]
    assert hit.tolist() == [0] and miss.tolist() == [3] and mg.tolist() == [5]
    rc, sg, sb, ss, ug = ora.bwd_segments(rows, bad_idx, off, 2)
    assert rc == ora.ERR_INDEX_RANGE and sg.tolist() == [0, 5] and sb.tolist() == [0, 3] and ss.tolist() == [0, 1, 2]
    neg = np.array([0, -1, 2, 1], dtype=np.int32)
    assert ora.histogram(rows, neg, off, 2)[0] == ora.ERR_INDEX_RANGE


# ------------------------------------------------------------------ hot / normal samples (Section III)
def test_classify_samples_brute_force_and_invariants(ora):
    for name, kw in (("tiny", {}), ("multi_hot", {"scale": 0.01})):
        wl = synth.workload(name, **kw)
        s, counts, hot, slot_of = _build(ora, wl)
        idx, off = s.batch(0)
        idx, off = idx.numpy(), off.numpy()
        rc, is_hot, hot_ids, normal_ids = ora.classify_samples(wl.rows, idx, off, wl.batch, slot_of)
        assert rc == 0
        # numpy special case: misses per sample via bincount over (bag mod B)
        gid = gids_of(wl, idx, off)
        sample = bag_of(off, idx.shape[0]) % wl.batch
        misses = np.bincount(sample, weights=(slot_of[gid] < 0), minlength=wl.batch)
        assert np.array_equal(is_hot, (misses == 0).astype(np.int32))
        assert hot_ids.size + normal_ids.size == wl.batch
        assert np.array_equal(hot_ids, np.nonzero(is_hot)[0]) and np.array_equal(normal_ids, np.nonzero(is_hot == 0)[0])
        assert 0 < hot_ids.size < wl.batch or name == "multi_hot"
        # extreme caches: everything cached -> all hot; nothing cached -> none hot (every sample has a lookup)
        rc, h_all, a, b = ora.classify_samples(wl.rows, idx, off, wl.batch, np.arange(wl.total_rows, dtype=np.int32))
        assert h_all.all() and b.size == 0
        rc, h_none, a, b = ora.classify_samples(wl.rows, idx, off, wl.batch, np.full(wl.total_rows, -1, dtype=np.int32))
        assert not h_none.any() and a.size == 0


def test_classify_samples_hand_case(ora):
    rows = [3, 2]
    B = 3
    #            table 0: sample0 [0,1]  sample1 []  sample2 [2]     table 1: sample0 [1]  sample1 []  sample2 [0]
    off = np.array([0, 2, 2, 3, 4, 4, 5], dtype=np.int32)
    idx = np.array([0, 1, 2, 1, 0], dtype=np.int32)
    slot_of = np.array([0, 1, -1, 2, 3], dtype=np.int32)      # only gid 2 (table 0 row 2) is not cached
    rc, is_hot, hot_ids, normal_ids = ora.classify_samples(rows, idx, off, B, slot_of)
    assert rc == 0 and is_hot.tolist() == [1, 1, 0]           # a sample without lookups needs no cold row: hot
    assert hot_ids.tolist() == [0, 1] and normal_ids.tolist() == [2]


# ------------------------------------------------------------------ coalescing (Section II-A)
def test_coalesce_matches_numpy_unique(ora):
    rng = np.random.default_rng(0)
    for n, hi in ((0, 5), (1, 5), (1000, 50), (5000, 10 ** 6)):
        mg = rng.integers(0, hi, n).astype(np.int32)
        rc, uq, inv = ora.coalesce(mg)
        assert rc == 0
        ref_u, ref_inv = np.unique(mg, return_inverse=True)
        assert np.array_equal(uq, ref_u) and np.array_equal(inv, ref_inv)
        assert np.array_equal(uq[inv], mg)                      # the list plus the indices reproduce every lookup


def test_coalesced_cost_matches_expected_communication(ora):
    # eq. (2)/(3): with nothing cached every lookup is a miss, and the coalesced transfer is the b indices plus
    # sum_e 1 - (1 - P(e))^b unique embeddings per feature
    wl = synth.workload("tiny", batch=4096)
    s = synth.Sampler(wl)
    idx, off = s.batch(0)
    none = np.full(wl.total_rows, -1, dtype=np.int32)
    rc, slot, hit, miss, mg = ora.remap(wl.rows, idx.numpy(), off.numpy(), wl.batch, none)
    assert miss.size == idx.numel()                             # eq. (4): b * d lookups communicated without coalescing
    rc, uq, inv = ora.coalesce(mg)
    EU = sum(float(np.sum(1.0 - (1.0 - s.row_probs(t).numpy()) ** wl.batch)) for t in range(wl.num_tables))
    assert abs(uq.size - EU) < 5 * math.sqrt(EU)
    assert uq.size < 0.5 * miss.size                            # Zipf 1.05 at b = 4096: coalescing more than halves it


# ------------------------------------------------------------------ cache use by portion (Fig. 4)
def test_portion_usage_brute_force(ora):
    wl = synth.workload("multi_hot", scale=0.01)
    s, counts, hot, slot_of = _build(ora, wl)
    idx, off = s.batch(0)
    idx, off = idx.numpy(), off.numpy()
    k = hot.size
    portion, nport = max(1, k // 4), 4
    rc, usage = ora.portion_usage(wl.rows, idx, off, wl.batch, slot_of, portion, nport)
    assert rc == 0
    gid = gids_of(wl, idx, off)
    sample = bag_of(off, idx.shape[0]) % wl.batch
    sl = slot_of[gid]
    ok = (sl >= 0) & (sl // portion < nport)
    pairs = np.unique(np.stack([sample[ok], sl[ok] // portion], 1), axis=0)      # distinct (sample, portion)
    assert np.array_equal(usage, np.bincount(pairs[:, 1], minlength=nport))
    assert usage.max() <= wl.batch
    assert usage[0] >= usage[-1]                 # slots are in hotness order: the first portion is used most


def test_partition_batch_brute_force_and_invariants(ora):
    """Sub-batch of selected samples (Section III): python-list brute force; hot and normal sub-batches together hold
    every lookup once; the forward sums of a sub-batch are the selected rows of the full batch's sums (bit for bit:
    same lookups, same order); a hot sub-batch has no miss."""
    wl = synth.workload("tiny", batch=97, bag_lambda=0.7)      # 1 + Poisson(0.7) lookups per bag, four tables
    s = synth.Sampler(wl)
    idx, off = (a.numpy() for a in s.batch(0))
    T, B = wl.num_tables, wl.batch
    rc, counts = ora.histogram(wl.rows, *(a.numpy() for a in s.batch(1, True)), B)
    k = wl.total_rows // 4
    rc, hot, slot_of = ora.hot_set(counts, k)
    rc, is_hot, hot_ids, normal_ids = ora.classify_samples(wl.rows, idx, off, B, slot_of)
    assert rc == 0 and 0 < hot_ids.size < B
    subs = {}
    for name, ids in (("hot", hot_ids), ("normal", normal_ids), ("all", np.arange(B, dtype=np.int32)),
                      ("none", np.zeros(0, dtype=np.int32))):
        rc, si, so = ora.partition_batch(T, idx, off, B, ids)
        assert rc == 0
        want_i, want_o = [], [0]
        for t in range(T):
            for j in ids:
                g = t * B + int(j)
                want_i += idx[off[g]:off[g + 1]].tolist()
                want_o.append(len(want_i))
        assert si.tolist() == want_i and so.tolist() == want_o
        subs[name] = (si, so, ids)
    assert np.array_equal(subs["all"][0], idx) and np.array_equal(subs["all"][1], off)
    assert subs["hot"][0].size + subs["normal"][0].size == idx.size
    tables = [t.numpy() for t in synth.make_tables_cpu(wl)]
    rc, full = ora.embedding_bag_fwd(wl.rows, tables, idx, off, B)
    for name in ("hot", "normal"):
        si, so, ids = subs[name]
        rc, out = ora.embedding_bag_fwd(wl.rows, tables, si, so, ids.size)
        sel = (np.arange(T)[:, None] * B + ids[None, :]).reshape(-1)
        assert rc == 0 and np.array_equal(out, full[sel])
    rc, slot, hit, miss, mg = ora.remap(wl.rows, subs["hot"][0], subs["hot"][1], hot_ids.size, slot_of)
    assert rc == 0 and miss.size == 0
    # refused: ids not ascending, out of range
    assert ora.partition_batch(T, idx, off, B, np.array([3, 3], dtype=np.int32))[0] != 0
    assert ora.partition_batch(T, idx, off, B, np.array([B], dtype=np.int32))[0] != 0
