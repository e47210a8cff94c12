"""Parity of the HIP path (through the C ABI) against the CPU oracle, element by element.

Integer outputs bit-exact; fp32 outputs within 1e-5 relative / 1e-6 absolute; bf16 rows within the admissible
rounding interval.  Sizes span several tiles of every kernel (2048-lookup compaction tiles, 4096-pair sort
tiles, 32-lookup reduce chunks) and end in ragged tails.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import oracle
from paper_2411_01611_amd import binding, synth
from gpu_harness import GpuCase, assert_bf16_within, assert_close
from util import gids_of

CASES = {
    "tiny": ("tiny", {}),
    "dlrm_small": ("dlrm_onehot", {"scale": 0.004, "batch": 1500}),
    "multi_hot_small": ("multi_hot", {"scale": 0.004, "batch": 333}),
    "low_skew_bf16": ("low_skew", {"scale": 0.002, "batch": 700}),
    "low_skew_uniform_bf16": ("low_skew_uniform", {"scale": 0.002, "batch": 257}),
    "host_spill_small": ("host_spill", {"scale": 0.0005, "batch": 3000}),
}


def _wl(case):
    name, kw = CASES[case]
    return synth.workload(name, **kw)


def _say(*a):
    print(*a, flush=True)


# "/scan": the same case with the separate scan kernels of the compactions forced (by default so few tiles add up
# their counts in the writing kernels)
# "/presort": remap starts the backward pass's sort on the library's side stream
# "/small": the caller states that no table gets more than 4096 lookups per batch, so the backward pass sorts each
#           table's pairs in LDS (one workgroup per table)
# "/apart": long runs and the other rows updated by two launches (by default they share one), and the backward
#           pass's (row, bag) pairs built by the backward pass (by default remap writes them)
VARIANTS = list(CASES) + ["tiny/apart", "multi_hot_small/apart", "dlrm_small/apart", "low_skew_bf16/apart",
                          "tiny/scan", "multi_hot_small/scan", "host_spill_small/scan", "low_skew_bf16/scan",
                          "tiny/presort", "multi_hot_small/presort", "host_spill_small/presort", "low_skew_bf16/presort",
                          "dlrm_small/presort",
                          "tiny/small", "dlrm_small/small", "host_spill_small/small", "low_skew_uniform_bf16/small"]


@pytest.fixture(params=VARIANTS)
def case(request):
    _say("case", request.param)
    name, _, variant = request.param.partition("/")
    c = GpuCase(_wl(name))
    if variant == "scan":
        c.s.set_tuning(binding.TUNE_FUSED_SCAN_MAX_TILES, 0)
    if variant == "presort":
        c.s.set_tuning(binding.TUNE_PRESORT, 1)
    if variant == "small":
        off = c.batch[1].numpy()
        per_table = np.diff(off[:: c.wl.batch])
        assert per_table.size == c.wl.num_tables and 0 < per_table.max() <= 4096
        c.s.set_tuning(binding.TUNE_MAX_TABLE_LOOKUPS, 4096)
    if variant == "apart":
        c.s.set_tuning(binding.TUNE_FUSED_LONG_MAX_L, 0)
        c.s.set_tuning(binding.TUNE_PAIRS_IN_REMAP, 0)
        c.s.set_tuning(binding.TUNE_UPDATE_MAX_BLOCKS, 7)      # the update kernel strides over the rows
    yield c
    c.close()


def test_build_cache_parity(case):
    counts, hot, slot_of = case.build()
    s = case.s
    assert s.sync_status() == 0
    assert s.cache_rows() == case.k
    assert np.array_equal(s.counts().cpu().numpy().view(np.uint32), counts)
    assert np.array_equal(s.hot_gid().cpu().numpy(), hot)
    assert np.array_equal(s.slot_of().cpu().numpy(), slot_of)
    rows = np.concatenate(case.ora_tables)
    cache = s.cache().cpu()
    cache = cache.numpy() if case.wl.dtype == "f32" else cache.view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(cache, rows[hot])


def test_remap_parity(case):
    case.build()
    wl = case.wl
    idx, off = case.batch
    rc, slot, hit, miss, mg = oracle.remap(wl.rows, idx.numpy(), off.numpy(), wl.batch, case.ora_slot_of)
    assert rc == 0
    rm = case.s.remap(*case.dev_batch(), wl.batch)
    assert case.s.sync_status() == 0
    n = rm.n_hit_miss.cpu().numpy()
    L = idx.numel()
    assert n.tolist() == [hit.size, miss.size] and hit.size + miss.size == L
    assert np.array_equal(rm.slot.cpu().numpy()[:L], slot)
    assert np.array_equal(rm.gid.cpu().numpy()[:L], gids_of(wl, idx.numpy(), off.numpy()))
    assert np.array_equal(rm.hit_pos.cpu().numpy()[: hit.size], hit)
    assert np.array_equal(rm.miss_pos.cpu().numpy()[: miss.size], miss)
    assert np.array_equal(rm.miss_gid.cpu().numpy()[: miss.size], mg)
    loc = np.where(slot >= 0, slot, 0)
    loc[miss] = case.k + np.arange(miss.size)
    assert np.array_equal(rm.loc.cpu().numpy()[:L], loc)


def test_fwd_parity(case):
    case.build()
    wl = case.wl
    idx, off = case.batch
    rc, want = oracle.embedding_bag_fwd(wl.rows, case.ora_tables, idx.numpy(), off.numpy(), wl.batch)
    assert rc == 0
    d_idx, d_off = case.dev_batch()
    rm = case.s.remap(d_idx, d_off, wl.batch)
    out = case.s.embedding_bag_fwd(d_idx, d_off, wl.batch, rm)
    assert case.s.sync_status() == 0
    assert_close(out.cpu().numpy(), want, "pooled output")
    # determinism: a second run is bit-identical
    out2 = case.s.embedding_bag_fwd(d_idx, d_off, wl.batch, rm)
    assert torch.equal(out, out2)


def _bwd_both(case, want_segments=True):
    wl = case.wl
    idx, off = case.batch
    grad = case.sampler.grads(0)
    lr, eps = np.float32(wl.lr), np.float32(wl.eps if wl.optimizer == "adagrad" else 0.0)
    opt = 1 if wl.optimizer == "adagrad" else 0
    rc, sg, sb, ss, ug = oracle.bwd_segments(wl.rows, idx.numpy(), off.numpy(), wl.batch)
    assert rc == 0
    rc, nr, ns, gr = oracle.embedding_bag_bwd_update(wl.rows, case.ora_tables, case.ora_state, opt, idx.numpy(),
                                                     off.numpy(), wl.batch, grad.numpy(), lr, eps, report=True,
                                                     n_unique=ug.size)
    assert rc == 0
    before = np.concatenate(case.ora_tables).copy()
    (rc,) = oracle.embedding_bag_bwd_update(wl.rows, case.ora_tables, case.ora_state, opt, idx.numpy(), off.numpy(),
                                            wl.batch, grad.numpy(), lr, eps)
    assert rc == 0
    d_idx, d_off = case.dev_batch()
    rm = case.s.remap(d_idx, d_off, wl.batch)
    bo = case.s.new_bwd_out(idx.numel()) if want_segments else None
    case.s.embedding_bag_bwd_update(d_idx, d_off, wl.batch, rm, grad.to(case.dev), float(lr), float(eps), bo)
    case.s.flush_cache()
    assert case.s.sync_status() == 0
    return (sg, sb, ss, ug), (nr, ns), before, bo


def test_bwd_parity(case):
    case.build()
    wl = case.wl
    (sg, sb, ss, ug), (nr, ns), before, bo = _bwd_both(case)
    U, nv = bo.n_unique.cpu().numpy().tolist()
    assert U == ug.size and nv == sg.size
    assert np.array_equal(bo.sorted_gid.cpu().numpy()[:nv], sg)
    assert np.array_equal(bo.sorted_bag.cpu().numpy()[:nv], sb)
    assert np.array_equal(bo.seg_start.cpu().numpy()[: U + 1], ss)
    assert np.array_equal(bo.unique_gid.cpu().numpy()[:U], ug)
    got = case.pinned_rows()
    want = np.concatenate(case.ora_tables)
    touched = np.zeros(wl.total_rows, dtype=bool)
    touched[ug] = True
    assert np.array_equal(got[~touched], before[~touched]), "rows without a lookup must not change"
    if wl.dtype == "f32":
        assert_close(got, want, "updated rows")
    else:
        assert_bf16_within(got[ug], nr, "updated bf16 rows")
    if wl.optimizer == "adagrad":
        assert_close(case.pinned_state_rows(), np.concatenate(case.ora_state), "adagrad accumulators")


def test_bwd_without_segment_outputs_gives_same_rows(case):
    case.build()
    _, _, _, bo = _bwd_both(case, want_segments=False)
    assert bo is None
    got = case.pinned_rows()
    if case.wl.dtype == "f32":
        assert_close(got, np.concatenate(case.ora_tables), "updated rows")


@pytest.mark.parametrize("name", ["tiny", "multi_hot_small", "low_skew_bf16"])
def test_source_invariance_across_budgets(name):
    """Pooled sums and post-flush tables are identical whether rows come from the cache or the host:
    budget 0 (every lookup misses), the workload's budget, and a budget that caches every row."""
    wl = _wl(name)
    outs, tabs, hits = [], [], []
    for budget in (0, wl.budget_bytes, wl.total_rows * wl.row_bytes + 5):
        _say("budget", budget)
        c = GpuCase(wl, budget_bytes=budget)
        c.build()
        d_idx, d_off = c.dev_batch()
        rm = c.s.remap(d_idx, d_off, wl.batch)
        out = c.s.embedding_bag_fwd(d_idx, d_off, wl.batch, rm)
        grad = c.sampler.grads(0).to(c.dev)
        c.s.embedding_bag_bwd_update(d_idx, d_off, wl.batch, rm, grad, wl.lr, wl.eps)
        c.s.flush_cache()
        assert c.s.sync_status() == 0
        outs.append(out.cpu())
        tabs.append(c.pinned_rows().copy())
        hits.append(rm.n_hit_miss.cpu().tolist())
        c.close()
    assert hits[0][0] == 0 and hits[2][1] == 0 and hits[1][0] > 0 and hits[1][1] > 0
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])
    assert np.array_equal(tabs[0], tabs[1]) and np.array_equal(tabs[0], tabs[2])


def test_onehot_forward_is_exact_gather():
    wl = _wl("tiny")
    c = GpuCase(wl)
    c.build()
    d_idx, d_off = c.dev_batch()
    out = c.s.embedding_bag_fwd(d_idx, d_off, wl.batch, c.s.remap(d_idx, d_off, wl.batch)).cpu().numpy()
    idx = c.batch[0].numpy()
    for t in range(wl.num_tables):
        assert np.array_equal(out[t * wl.batch:(t + 1) * wl.batch], c.ora_tables[t][idx[t * wl.batch:(t + 1) * wl.batch]])
    c.close()


def test_two_steps_in_a_row_match_oracle():
    """Second step reads rows the first step updated (cache for hot rows, host for cold ones)."""
    wl = _wl("multi_hot_small")
    c = GpuCase(wl)
    c.build()
    opt = 1
    for step in range(2):
        idx, off = c.sampler.batch(step)
        grad = c.sampler.grads(step)
        rc, want = oracle.embedding_bag_fwd(wl.rows, c.ora_tables, idx.numpy(), off.numpy(), wl.batch)
        oracle.embedding_bag_bwd_update(wl.rows, c.ora_tables, c.ora_state, opt, idx.numpy(), off.numpy(), wl.batch,
                                        grad.numpy(), np.float32(wl.lr), np.float32(wl.eps))
        d_idx, d_off = idx.to(c.dev), off.to(c.dev)
        rm = c.s.remap(d_idx, d_off, wl.batch)
        out = c.s.embedding_bag_fwd(d_idx, d_off, wl.batch, rm)
        assert_close(out.cpu().numpy(), want, f"step {step} output")
        c.s.embedding_bag_bwd_update(d_idx, d_off, wl.batch, rm, grad.to(c.dev), wl.lr, wl.eps)
    c.s.flush_cache()
    assert c.s.sync_status() == 0
    assert_close(c.pinned_rows(), np.concatenate(c.ora_tables), "rows after two steps")
    assert_close(c.pinned_state_rows(), np.concatenate(c.ora_state), "state after two steps")
    c.close()


def test_classify_samples_parity(case):
    """Hot / normal samples: flags and both id lists bit-exact, n_hot + n_normal = B."""
    case.build()
    wl = case.wl
    idx, off = case.batch
    rc, is_hot, hot_ids, normal_ids = oracle.classify_samples(wl.rows, idx.numpy(), off.numpy(), wl.batch, case.ora_slot_of)
    assert rc == 0
    d_idx, d_off = case.dev_batch()
    rm = case.s.remap(d_idx, d_off, wl.batch)
    co = case.s.classify_samples(d_idx, d_off, wl.batch, rm)
    assert case.s.sync_status() == 0
    nh, nn = co.n_hot_normal.cpu().tolist()
    assert nh + nn == wl.batch and nh == hot_ids.size
    assert np.array_equal(co.is_hot.cpu().numpy()[: wl.batch], is_hot)
    assert np.array_equal(co.hot_ids.cpu().numpy()[:nh], hot_ids)
    assert np.array_equal(co.normal_ids.cpu().numpy()[:nn], normal_ids)


def test_classify_samples_extreme_budgets():
    wl = _wl("multi_hot_small")
    for budget, all_hot in ((0, False), (wl.total_rows * wl.row_bytes, True)):
        c = GpuCase(wl, budget_bytes=budget)
        c.build()
        d_idx, d_off = c.dev_batch()
        co = c.s.classify_samples(d_idx, d_off, wl.batch, c.s.remap(d_idx, d_off, wl.batch))
        nh, nn = co.n_hot_normal.cpu().tolist()
        assert (nh, nn) == ((wl.batch, 0) if all_hot else (0, wl.batch))
        c.close()


def test_coalesced_remap_and_forward(case):
    """Section II-A coalescing: distinct missed rows listed once (bit-exact against the oracle), every missed
    lookup pointing into that list; forward and the following backward give the same values as without it."""
    case.build()
    wl = case.wl
    idx, off = case.batch
    rc, slot, hit, miss, mg = oracle.remap(wl.rows, idx.numpy(), off.numpy(), wl.batch, case.ora_slot_of)
    rc, uq, inv = oracle.coalesce(mg)
    assert rc == 0
    d_idx, d_off = case.dev_batch()
    L = idx.numel()
    plain = case.s.remap(d_idx, d_off, wl.batch)
    out_plain = case.s.embedding_bag_fwd(d_idx, d_off, wl.batch, plain)
    rm = case.s.remap(d_idx, d_off, wl.batch, coalesce=True)
    assert case.s.sync_status() == 0
    assert rm.n_unique_miss.cpu().tolist() == [uq.size, miss.size]
    assert np.array_equal(rm.unique_miss_gid.cpu().numpy()[: uq.size], uq)
    loc = rm.loc.cpu().numpy()[:L]
    assert np.array_equal(loc[miss], case.k + inv)
    assert np.array_equal(loc[hit], slot[hit])
    assert np.array_equal(rm.miss_gid.cpu().numpy()[: miss.size], mg)       # the per-lookup lists are unchanged
    out = case.s.embedding_bag_fwd(d_idx, d_off, wl.batch, rm)
    assert torch.equal(out, out_plain)
    rc, want = oracle.embedding_bag_fwd(wl.rows, case.ora_tables, idx.numpy(), off.numpy(), wl.batch)
    assert_close(out.cpu().numpy(), want, "pooled output with coalesced misses")
    # backward right after this forward takes cold rows from the coalesced staging area
    grad = case.sampler.grads(0)
    lr, eps = np.float32(wl.lr), np.float32(wl.eps if wl.optimizer == "adagrad" else 0.0)
    opt = 1 if wl.optimizer == "adagrad" else 0
    rc, sg, sb, ss, ug = oracle.bwd_segments(wl.rows, idx.numpy(), off.numpy(), wl.batch)
    rc, nr, ns, gr = oracle.embedding_bag_bwd_update(wl.rows, case.ora_tables, case.ora_state, opt, idx.numpy(),
                                                     off.numpy(), wl.batch, grad.numpy(), lr, eps, report=True,
                                                     n_unique=ug.size)
    oracle.embedding_bag_bwd_update(wl.rows, case.ora_tables, case.ora_state, opt, idx.numpy(), off.numpy(), wl.batch,
                                    grad.numpy(), lr, eps)
    case.s.embedding_bag_bwd_update(d_idx, d_off, wl.batch, rm, grad.to(case.dev), float(lr), float(eps))
    case.s.flush_cache()
    assert case.s.sync_status() == 0
    if wl.dtype == "f32":
        assert_close(case.pinned_rows(), np.concatenate(case.ora_tables), "rows after coalesced step")
    else:
        assert_bf16_within(case.pinned_rows()[ug], nr, "bf16 rows after coalesced step")


def test_coalescing_without_cache_matches_expected_unique():
    """No cache at all (the paper's coalescing-only setting): every lookup misses and the staged rows are the
    batch's distinct rows."""
    wl = _wl("host_spill_small")
    c = GpuCase(wl, budget_bytes=0)
    c.build()
    d_idx, d_off = c.dev_batch()
    rm = c.s.remap(d_idx, d_off, wl.batch, coalesce=True)
    U, n_miss = rm.n_unique_miss.cpu().tolist()
    gid = gids_of(wl, c.batch[0].numpy(), c.batch[1].numpy())
    assert n_miss == gid.size and U == np.unique(gid).size and U < 0.6 * n_miss
    out = c.s.embedding_bag_fwd(d_idx, d_off, wl.batch, rm)
    rc, want = oracle.embedding_bag_fwd(wl.rows, c.ora_tables, c.batch[0].numpy(), c.batch[1].numpy(), wl.batch)
    assert_close(out.cpu().numpy(), want, "coalesced forward without a cache")
    c.close()


def test_portion_usage_parity(case):
    case.build()
    wl = case.wl
    idx, off = case.batch
    portion, nport = max(1, case.k // 5), 7           # the last portions lie beyond the cache: zero use
    rc, want = oracle.portion_usage(wl.rows, idx.numpy(), off.numpy(), wl.batch, case.ora_slot_of, portion, nport)
    assert rc == 0
    d_idx, d_off = case.dev_batch()
    rm = case.s.remap(d_idx, d_off, wl.batch)
    got = case.s.portion_usage(d_idx, d_off, wl.batch, rm, portion, nport)
    assert case.s.sync_status() == 0
    assert np.array_equal(got.cpu().numpy(), want)


# ---- budget chooser: eq. (6)/(7) on the device skew table -------------------------------------------------
def _plan_params(case, frac):
    """M holds `frac` of the rows next to a batch; a makes the batch a few thousand samples when nothing is cached."""
    wl = case.wl
    d = float(wl.dim)
    M = wl.total_rows * d * frac
    a = M / 4096.0
    return M, a, d, 1.0e6, len(case.profile) * wl.batch


@pytest.mark.parametrize("frac", [0.3, 2.0])
def test_epoch_cost_parity(case, frac):
    counts, _, _ = case.build()
    wl = case.wl
    M, a, d, Q, S = _plan_params(case, frac)
    kf = int(min(wl.total_rows, (M - a) // d))
    for k in sorted({0, 1, case.k, kf // 2, kf}):
        _say("epoch_cost", wl.name, "k", k)
        rc, want, b_want = oracle.epoch_cost(wl.num_tables, counts, S, k, M, a, d, Q)
        assert rc == 0
        got, b = case.s.epoch_cost(M, a, Q, S, k)
        assert abs(b - b_want) <= 1e-12 * b_want
        assert abs(got - want) <= 1e-10 * want            # same fp64 terms, summed per count class instead of per row
    if kf < wl.total_rows:                                # one row more leaves no room for a sample: refused by both
        assert oracle.epoch_cost(wl.num_tables, counts, S, kf + 1, M, a, d, Q)[0] != 0
        with pytest.raises(binding.ScarsError):
            case.s.epoch_cost(M, a, Q, S, kf + 1)


def test_plan_cache_matches_brute_force():
    # a table small enough that the oracle can try every k; the library examines every k as well
    wl = synth.workload("tiny", rows=(1500, 900, 600), budget_bytes=1 << 16)
    c = GpuCase(wl, nprofile=8)
    counts, _, _ = c.build()
    for frac in (0.2, 0.6, 3.0):
        M, a, d, Q, S = _plan_params(c, frac)
        a = M / 512.0
        kf = int(min(wl.total_rows, (M - a) // d))
        _say("plan_cache", "frac", frac, "k_max", kf)
        rc, bk, bc = oracle.plan_brute(wl.num_tables, counts, S, kf, M, a, d, Q)
        assert rc == 0
        p = c.s.plan_cache(M, a, Q, S)
        assert p["k_max"] == kf
        assert abs(p["best_cost"] - bc) <= 1e-10 * bc
        if p["best_k"] != bk:                             # only a tie up to summation order may move the argmin
            assert abs(oracle.epoch_cost(wl.num_tables, counts, S, int(p["best_k"]), M, a, d, Q)[1] - bc) <= 1e-10 * bc
        rc, c0, b0 = oracle.epoch_cost(wl.num_tables, counts, S, 0, M, a, d, Q)
        assert abs(p["cost_no_cache"] - c0) <= 1e-10 * c0 and abs(p["batch_no_cache"] - b0) <= 1e-12 * b0
        assert abs(p["best_batch"] - (M - p["best_k"] * d) / a) <= 1e-9
    c.close()


def test_plan_cache_grid_search_is_no_worse_than_sampled_k(case):
    # beyond 4096 candidate rows the search is a narrowing grid: its result must not lose to any k the oracle samples
    counts, _, _ = case.build()
    wl = case.wl
    M, a, d, Q, S = _plan_params(case, 0.5)
    p = case.s.plan_cache(M, a, Q, S)
    rc, want, _ = oracle.epoch_cost(wl.num_tables, counts, S, int(p["best_k"]), M, a, d, Q)
    assert rc == 0 and abs(p["best_cost"] - want) <= 1e-10 * want
    kf = int(p["k_max"])
    for k in np.unique(np.linspace(0, kf, 41).astype(np.int64)):
        rc, ck, _ = oracle.epoch_cost(wl.num_tables, counts, S, int(k), M, a, d, Q)
        assert rc == 0 and p["best_cost"] <= ck * (1 + 1e-10)


def test_epoch_cost_with_counts_beyond_the_binned_range():
    # counts written straight into the device skew table: many rows of one small count (the one-atomic-per-wave
    # path), rows in the globally binned range, and rows whose count exceeds 65535 (kept as a list)
    wl = synth.workload("tiny", rows=(7000, 3000))
    c = GpuCase(wl, nprofile=1)
    N = wl.total_rows
    u = synth.uniform01(synth.stream_key(wl.seed, 77), torch.arange(N, dtype=torch.int64)).numpy()
    counts = np.where(u < 0.7, 3, np.where(u < 0.9, (u * 60000).astype(np.int64), (u * 3.0e6).astype(np.int64))).astype(np.uint32)
    counts[:640] = 0
    assert (counts >= 65536).sum() > 100 and ((counts >= 2048) & (counts < 65536)).sum() > 100
    c.s.counts().copy_(torch.from_numpy(counts.view(np.int32)))
    S, d, Q = 4_000_000, float(wl.dim), 1.0e6
    M = N * d * 0.5
    a = M / 1000.0
    for k in (0, 5, 800, 3000):
        rc, want, _ = oracle.epoch_cost(wl.num_tables, counts, S, k, M, a, d, Q)
        assert rc == 0
        got, _ = c.s.epoch_cost(M, a, Q, S, k)
        assert abs(got - want) <= 1e-10 * want
    c.close()


# ---- backward sort started by remap on the library's side stream -------------------------------------------
def _room(wl):
    """Lookups to bind for: well above any batch the sampler draws."""
    return int(wl.num_bags * (1.0 + (wl.bag_lambda or 0.0)) * 1.3) + 1024


def _presort_steps(c, steps, budget_note):
    """steps x (remap, forward, backward without segment outputs) on both sides; rows compared after a flush."""
    wl = c.wl
    opt = 1 if wl.optimizer == "adagrad" else 0
    lr, eps = np.float32(wl.lr), np.float32(wl.eps if opt else 0.0)
    for step in range(steps):
        idx, off = c.sampler.batch(step)
        grad = c.sampler.grads(step)
        rc, want = oracle.embedding_bag_fwd(wl.rows, c.ora_tables, idx.numpy(), off.numpy(), wl.batch)
        assert rc == 0
        (rc,) = oracle.embedding_bag_bwd_update(wl.rows, c.ora_tables, c.ora_state, opt, idx.numpy(), off.numpy(), wl.batch,
                                                grad.numpy(), lr, eps)
        assert rc == 0
        d_idx, d_off = idx.to(c.dev), off.to(c.dev)
        rm = c.s.remap(d_idx, d_off, wl.batch)
        out = c.s.embedding_bag_fwd(d_idx, d_off, wl.batch, rm)
        c.s.embedding_bag_bwd_update(d_idx, d_off, wl.batch, rm, grad.to(c.dev), float(lr), float(eps))
        if wl.dtype == "f32":
            assert_close(out.cpu().numpy(), want, f"{budget_note} step {step} output")
    c.s.flush_cache()
    assert c.s.sync_status() == 0
    if wl.dtype == "f32":
        assert_close(c.pinned_rows(), np.concatenate(c.ora_tables), f"{budget_note} rows")
        if opt:
            assert_close(c.pinned_state_rows(), np.concatenate(c.ora_state), f"{budget_note} accumulators")


@pytest.mark.parametrize("name", ["tiny", "multi_hot_small", "host_spill_small", "dlrm_small"])
@pytest.mark.parametrize("budget", ["own", "none", "all"])
def test_presort_steps_match_oracle(name, budget):
    wl = _wl(name)
    bb = {"own": None, "none": 0, "all": wl.total_rows * wl.row_bytes}[budget]
    _say("presort", name, budget)
    c = GpuCase(wl, budget_bytes=bb, max_L=_room(wl))
    c.s.set_tuning(binding.TUNE_PRESORT, 1)
    c.build()
    _presort_steps(c, 3, f"{name}/{budget}")
    # every backward pass used the prepared segments; with every row cached nothing is prepared (no link to hide behind)
    assert c.s.get_counter(binding.COUNTER_PREPARED_USED) == (0 if budget == "all" else 3)
    c.close()


def test_presort_falls_back_when_the_calls_do_not_line_up():
    """The prepared segments are used only for remap -> forward -> backward of one batch without segment outputs;
    every other order sorts again and gives the same rows."""
    wl = _wl("multi_hot_small")
    c = GpuCase(wl, max_L=_room(wl))
    c.s.set_tuning(binding.TUNE_PRESORT, 1)
    c.build()
    opt, lr, eps = 1, np.float32(wl.lr), np.float32(wl.eps)
    used = lambda: c.s.get_counter(binding.COUNTER_PREPARED_USED)

    def oracle_step(step):
        idx, off = c.sampler.batch(step)
        (rc,) = oracle.embedding_bag_bwd_update(wl.rows, c.ora_tables, c.ora_state, opt, idx.numpy(), off.numpy(), wl.batch,
                                                c.sampler.grads(step).numpy(), lr, eps)
        assert rc == 0
        return idx.to(c.dev), off.to(c.dev), c.sampler.grads(step).to(c.dev)

    # (1) backward without a forward pass: cold rows must come from the host, not from a stale staging area
    i0, o0, g0 = oracle_step(0)
    rm = c.s.remap(i0, o0, wl.batch)
    c.s.embedding_bag_bwd_update(i0, o0, wl.batch, rm, g0, float(lr), float(eps))
    assert used() == 0
    # (2) segment outputs requested: sorted in line, outputs bit-exact
    i1, o1, g1 = oracle_step(1)
    rc, sg, sb, ss, ug = oracle.bwd_segments(wl.rows, i1.cpu().numpy(), o1.cpu().numpy(), wl.batch)
    rm = c.s.remap(i1, o1, wl.batch)
    c.s.embedding_bag_fwd(i1, o1, wl.batch, rm)
    bo = c.s.new_bwd_out(i1.numel())
    c.s.embedding_bag_bwd_update(i1, o1, wl.batch, rm, g1, float(lr), float(eps), bo)
    assert used() == 0
    assert np.array_equal(bo.unique_gid.cpu().numpy()[: ug.size], ug) and np.array_equal(bo.seg_start.cpu().numpy()[: ug.size + 1], ss)
    # (3) two remaps, then the step of the second batch with other output arrays than the first
    i2, o2, g2 = oracle_step(2)
    rm_a = c.s.remap(i0, o0, wl.batch)
    rm_b = c.s.remap(i2, o2, wl.batch, c.s.new_remap_out())
    c.s.embedding_bag_fwd(i2, o2, wl.batch, rm_b)
    c.s.embedding_bag_bwd_update(i2, o2, wl.batch, rm_b, g2, float(lr), float(eps))
    assert used() == 1
    # (4) a step whose backward pass is given the first remap's arrays: they describe another batch's preparation
    i3, o3, g3 = oracle_step(3)
    rm_c = c.s.remap(i3, o3, wl.batch, rm_a)
    c.s.embedding_bag_fwd(i3, o3, wl.batch, rm_c)
    c.s.remap(i2, o2, wl.batch, rm_b)                                   # prepares batch 2 again; batch 3's is gone
    c.s.embedding_bag_bwd_update(i3, o3, wl.batch, rm_c, g3, float(lr), float(eps))
    assert used() == 1
    c.s.flush_cache()
    assert c.s.sync_status() == 0
    assert_close(c.pinned_rows(), np.concatenate(c.ora_tables), "rows after mixed call orders")
    assert_close(c.pinned_state_rows(), np.concatenate(c.ora_state), "accumulators after mixed call orders")
    c.close()


# ---- sub-batches of hot and normal samples (Section III) ---------------------------------------------------------
@pytest.mark.parametrize("name,budget_frac", [("tiny", 0.25), ("dlrm_small", 0.3), ("multi_hot_small", 0.9),
                                              ("host_spill_small", 0.1), ("low_skew_bf16", 0.95)])
@pytest.mark.parametrize("scan", [False, True])
def test_partition_batch_parity_and_hot_subbatch_never_misses(name, budget_frac, scan):
    wl = _wl(name)
    c = GpuCase(wl, budget_bytes=int(wl.total_rows * budget_frac) * wl.row_bytes)
    if scan:
        c.s.set_tuning(binding.TUNE_FUSED_SCAN_MAX_TILES, 0)
    c.build()
    T, B = wl.num_tables, wl.batch
    idx, off = c.batch
    d_idx, d_off = c.dev_batch()
    rm = c.s.remap(d_idx, d_off, B)
    full = c.s.embedding_bag_fwd(d_idx, d_off, B, rm).clone()
    cls = c.s.classify_samples(d_idx, d_off, B, rm)
    rc, is_hot, hot_ids, normal_ids = oracle.classify_samples(wl.rows, idx.numpy(), off.numpy(), B, c.ora_slot_of)
    assert rc == 0
    _say("partition", name, "hot samples", hot_ids.size, "of", B)
    for which, ids_dev, ids_ref in ((0, cls.hot_ids, hot_ids), (1, cls.normal_ids, normal_ids)):
        rc, want_i, want_o = oracle.partition_batch(T, idx.numpy(), off.numpy(), B, ids_ref)
        assert rc == 0
        sub_i, sub_o, cnt = c.s.partition_batch(d_idx, d_off, B, ids_dev, cls.n_hot_normal[which:which + 1])
        assert c.s.sync_status() == 0
        n = ids_ref.size
        assert cnt.cpu().tolist() == [want_i.size, T * n]
        assert np.array_equal(sub_o.cpu().numpy()[: T * n + 1], want_o)
        assert np.array_equal(sub_i.cpu().numpy()[: want_i.size], want_i)
        if n == 0:
            continue
        # the sub-batch through the per-batch calls, with B = n
        s_idx, s_off = sub_i[: want_i.size].contiguous(), sub_o[: T * n + 1].contiguous()
        rm_s = c.s.remap(s_idx, s_off, n)
        out_s = c.s.embedding_bag_fwd(s_idx, s_off, n, rm_s)
        assert c.s.sync_status() == 0
        sel = (torch.arange(T)[:, None] * B + torch.from_numpy(ids_ref.astype(np.int64))[None, :]).reshape(-1).to(c.dev)
        assert torch.equal(out_s, full[sel]), "a sub-batch's sums are the selected rows of the batch's, bit for bit"
        if which == 0:
            assert rm_s.n_hit_miss.cpu().tolist() == [want_i.size, 0]      # a hot sub-batch never touches the host link
    c.close()


def test_partition_batch_of_nothing_and_of_everything():
    wl = _wl("multi_hot_small")
    c = GpuCase(wl)
    c.build()
    T, B = wl.num_tables, wl.batch
    idx, off = c.batch
    d_idx, d_off = c.dev_batch()
    ids = torch.arange(B, dtype=torch.int32, device=c.dev)
    for n in (0, B):
        nt = torch.tensor([n], dtype=torch.int32, device=c.dev)
        sub_i, sub_o, cnt = c.s.partition_batch(d_idx, d_off, B, ids, nt)
        assert c.s.sync_status() == 0
        if n == 0:
            assert cnt.cpu().tolist() == [0, 0] and int(sub_o[0]) == 0
        else:
            assert cnt.cpu().tolist() == [idx.numel(), T * B]
            assert torch.equal(sub_i[: idx.numel()].cpu(), idx) and torch.equal(sub_o.cpu(), off)
    c.close()


def test_caching_gain_parity(case):
    """eq. (11)/(12) from the device skew table against the oracle's per-row sums."""
    counts, _, _ = case.build()
    wl = case.wl
    M, a, d, Q, S = _plan_params(case, 0.5)
    kf = int(min(wl.total_rows - 1, (M - a - d) // d))
    for k in sorted({0, 1, case.k, kf // 2, kf}):
        rc, lhs, t1 = oracle.caching_gain(counts, S, k, M, a, d)
        assert rc == 0
        g_lhs, g_t1 = case.s.caching_gain(M, a, S, k)
        assert abs(g_lhs - lhs) <= 1e-12 and abs(g_t1 - t1) <= 1e-10 * max(1.0, abs(t1))
    with pytest.raises(binding.ScarsError):
        case.s.caching_gain(M, a, S, wl.total_rows)


@pytest.mark.parametrize("name", ["multi_hot_small", "host_spill_small"])
def test_twenty_steps_with_the_side_streams_match_oracle(name):
    """A longer run with every side-stream path on (sort started by remap, long runs beside the per-row kernel, cached
    bags pooled beside the fetch): rows and accumulators after twenty steps."""
    wl = _wl(name)
    c = GpuCase(wl, max_L=_room(wl))
    c.s.set_tuning(binding.TUNE_PRESORT, 1)
    c.build()
    _presort_steps(c, 20, f"{name}, twenty steps")
    assert c.s.get_counter(binding.COUNTER_PREPARED_USED) == 20
    c.close()
