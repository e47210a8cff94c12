"""Parity at the benchmark's full size and launch configuration (workload `multi_hot`: 8 tables x 5M rows x
dim 128 fp32, batch 4096, bags 1+Poisson(19), 2 GB cache, Adagrad), against the CPU oracle working on the same
pinned tables.  Tables and batches are generated on the GPU by the seeded generators (as bench.py does).

Checked: histogram and hot set bit-exact over all 40M rows; remap lists bit-exact; every pooled output within
tolerance; sorted segments bit-exact; every updated row and accumulator within tolerance after a flush;
rows without a lookup untouched (sampled); the step run again on the next batch, and a third time in bench.py's
launch configuration (backward sort started by remap on the side stream, no segment outputs).
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import oracle
from paper_2411_01611_amd import binding, synth
from gpu_harness import assert_close


def _say(*a):
    print(*a, flush=True)


@pytest.fixture(scope="module")
def full():
    dev = torch.device("cuda:0")
    wl = synth.workload("multi_hot")
    _say("allocating and filling", wl.total_rows * wl.row_bytes * 2 / 1e9, "GB pinned")
    tabs, state = [], []
    for t in range(wl.num_tables):
        p = binding.PinnedArray((wl.rows[t], wl.dim), np.float32)
        chunk = 1 << 20
        for r0 in range(0, wl.rows[t], chunk):
            r1 = min(wl.rows[t], r0 + chunk)
            p.copy_from_device(synth.row_values(wl, t, r0, r1, dev).contiguous(), r0)
            torch.cuda.synchronize()
        s = binding.PinnedArray((wl.rows[t], wl.dim), np.float32)
        s.np[...] = 0.0
        tabs.append(p)
        state.append(s)
    sc = binding.Scars(wl.rows, wl.dim, binding.DTYPE_F32, [p.ptr for p in tabs], binding.OPT_ADAGRAD,
                       [p.ptr for p in state])
    smp = synth.Sampler(wl, dev)
    yield wl, dev, tabs, state, sc, smp
    sc.close()
    for p in tabs + state:
        p.free()


@pytest.mark.timeout(900)
def test_full_size_path_matches_oracle(full):
    wl, dev, tabs, state, sc, smp = full
    P = 8                                                     # profile batches (5.2M lookups)
    prof = [smp.batch(p, True) for p in range(P)]
    batches = [smp.batch(e) for e in range(3)]
    max_L = max(int(b[0].numel()) for b in prof + batches)
    sc.bind_buffers(wl.budget_bytes, max_L, wl.num_bags)
    # ---- build_cache
    counts = np.zeros(wl.total_rows, dtype=np.uint32)
    sc.build_cache(None, None, 0, wl.budget_bytes, 0)
    for n, (idx, off) in enumerate(prof):
        rc, counts = oracle.histogram(wl.rows, idx.cpu().numpy(), off.cpu().numpy(), wl.batch, counts)
        assert rc == 0
        sc.build_cache(idx, off, wl.batch, wl.budget_bytes, 1 if n == P - 1 else 2)
    assert sc.sync_status() == 0
    _say("oracle hot set over", wl.total_rows, "rows")
    k = oracle.budget_rows(wl.total_rows, wl.row_bytes, wl.budget_bytes)
    assert k == 3_906_250 == sc.cache_rows()
    rc, hot, slot_of = oracle.hot_set(counts, k)
    assert np.array_equal(sc.counts().cpu().numpy().view(np.uint32), counts)
    assert np.array_equal(sc.hot_gid().cpu().numpy(), hot)
    assert np.array_equal(sc.slot_of().cpu().numpy(), slot_of)
    ora_tabs = [p.np for p in tabs]          # the oracle reads the same pinned tables, in report mode, before each GPU step
    sample = np.random.default_rng(0).integers(0, k, 4096)
    rb = wl.row_base
    got = sc.cache()[torch.from_numpy(sample).to(dev)].cpu().numpy()
    for j, s in enumerate(sample):
        g = int(hot[s]); t = int(np.searchsorted(rb, g, side="right") - 1)
        assert np.array_equal(got[j], ora_tabs[t][g - rb[t]])
    # ---- three steps; the last one in bench.py's launch configuration: remap also starts the backward pass's sort on
    # the library's side stream, and no segment outputs are requested
    lr, eps = np.float32(wl.lr), np.float32(wl.eps)
    for step, (idx, off) in enumerate(batches):
        _say("step", step)
        hi, ho = idx.cpu().numpy(), off.cpu().numpy()
        grad = smp.grads(step)
        hg = grad.cpu().numpy()
        rc, slot, hit, miss, mg = oracle.remap(wl.rows, hi, ho, wl.batch, slot_of)
        rc2, want = oracle.embedding_bag_fwd(wl.rows, ora_tabs, hi, ho, wl.batch)
        rc3, sg, sb, ss, ug = oracle.bwd_segments(wl.rows, hi, ho, wl.batch)
        rc4, nr, ns, gr = oracle.embedding_bag_bwd_update(wl.rows, ora_tabs, [p.np for p in state], 1, hi, ho, wl.batch,
                                                          hg, lr, eps, report=True, n_unique=ug.size)
        assert rc == rc2 == rc3 == rc4 == 0
        # untouched-row sample taken before the GPU step
        rng = np.random.default_rng(step + 1)
        probe = rng.integers(0, wl.total_rows, 20000)
        probe = probe[~np.isin(probe, ug)]
        pt = np.searchsorted(rb, probe, side="right") - 1
        before = np.stack([ora_tabs[t][g - rb[t]] for g, t in zip(probe[:2000], pt[:2000])])
        L = idx.numel()
        presort = step == 2
        sc.set_tuning(binding.TUNE_PRESORT, 131072 if presort else 0)
        rm = sc.remap(idx, off, wl.batch)
        out = sc.embedding_bag_fwd(idx, off, wl.batch, rm)
        bo = None if presort else sc.new_bwd_out(L)
        sc.embedding_bag_bwd_update(idx, off, wl.batch, rm, grad, float(lr), float(eps), bo)
        sc.flush_cache()
        assert sc.sync_status() == 0
        assert sc.get_counter(binding.COUNTER_PREPARED_USED) == (1 if presort else 0)
        assert rm.n_hit_miss.cpu().tolist() == [hit.size, miss.size] and hit.size + miss.size == L
        assert np.array_equal(rm.slot.cpu().numpy()[:L], slot)
        assert np.array_equal(rm.hit_pos.cpu().numpy()[: hit.size], hit)
        assert np.array_equal(rm.miss_pos.cpu().numpy()[: miss.size], miss)
        assert np.array_equal(rm.miss_gid.cpu().numpy()[: miss.size], mg)
        assert_close(out.cpu().numpy(), want, "pooled output at full size")
        if bo is not None:
            U, nv = bo.n_unique.cpu().tolist()
            assert U == ug.size and nv == sg.size
            assert np.array_equal(bo.sorted_gid.cpu().numpy()[:nv], sg)
            assert np.array_equal(bo.sorted_bag.cpu().numpy()[:nv], sb)
            assert np.array_equal(bo.seg_start.cpu().numpy()[: U + 1], ss)
            assert np.array_equal(bo.unique_gid.cpu().numpy()[:U], ug)
        # every touched row and accumulator (the pinned tables were updated in place by the GPU and flushed)
        ut = np.searchsorted(rb, ug, side="right") - 1
        for t in range(wl.num_tables):
            sel = ut == t
            rows_t = ug[sel] - rb[t]
            assert_close(tabs[t].np[rows_t], nr[sel].astype(np.float32), f"updated rows of table {t}")
            assert_close(state[t].np[rows_t], ns[sel].astype(np.float32), f"accumulators of table {t}")
        after = np.stack([ora_tabs[t][g - rb[t]] for g, t in zip(probe[:2000], pt[:2000])])
        assert np.array_equal(before, after), "rows without a lookup must not change"


@pytest.mark.timeout(900)
def test_full_size_look_ahead_steps_match_oracle(full):
    """The order bench.py's `lookahead` leg times, at its size: remap(next) -> bwd_update_ahead(this, next) ->
    fwd(next) over three consecutive batches.  Before each update the oracle computes, in report mode on the same
    pinned tables, what every touched row and accumulator must become; after it (and a flush) the tables are compared,
    and the next forward pass, part of whose rows were fetched while the update ran, is compared with the oracle's sums
    over the updated tables."""
    wl, dev, tabs, state, sc, smp = full
    prof = [smp.batch(p, True) for p in range(4)]
    batches = [smp.batch(e) for e in range(3, 6)]
    max_L = max(int(b[0].numel()) for b in prof + batches)
    sc.bind_buffers(wl.budget_bytes, max_L, wl.num_bags)
    sc.build_cache(None, None, 0, wl.budget_bytes, 0)
    for n, (idx, off) in enumerate(prof):
        sc.build_cache(idx, off, wl.batch, wl.budget_bytes, 1 if n == len(prof) - 1 else 2)
    sc.set_tuning(binding.TUNE_LOOKAHEAD, 1)
    sc.set_tuning(binding.TUNE_PRESORT, 131072)
    used0 = sc.get_counter(binding.COUNTER_AHEAD_USED)
    ora_tabs, ora_state = [p.np for p in tabs], [p.np for p in state]
    lr, eps = np.float32(wl.lr), np.float32(wl.eps)
    rb = wl.row_base
    rms = [sc.new_remap_out(max_L), sc.new_remap_out(max_L)]
    host = [(i.cpu().numpy(), o.cpu().numpy()) for i, o in batches]
    sc.remap(batches[0][0], batches[0][1], wl.batch, rms[0])
    out = sc.embedding_bag_fwd(batches[0][0], batches[0][1], wl.batch, rms[0])
    rc, want = oracle.embedding_bag_fwd(wl.rows, ora_tabs, host[0][0], host[0][1], wl.batch)
    assert rc == 0
    assert_close(out.cpu().numpy(), want, "first forward pass")
    for e in range(2):
        _say("look-ahead step", e)
        (idx, off), (nidx, noff) = batches[e], batches[e + 1]
        grad = smp.grads(e)
        rc, sg, sb, ss, ug = oracle.bwd_segments(wl.rows, host[e][0], host[e][1], wl.batch)
        rc2, nr, ns, gr = oracle.embedding_bag_bwd_update(wl.rows, ora_tabs, ora_state, 1, host[e][0], host[e][1], wl.batch,
                                                          grad.cpu().numpy(), lr, eps, report=True, n_unique=ug.size)
        assert rc == rc2 == 0
        sc.remap(nidx, noff, wl.batch, rms[(e + 1) % 2])
        sc.embedding_bag_bwd_update_ahead(idx, off, wl.batch, rms[e % 2], grad, float(lr), float(eps), rms[(e + 1) % 2],
                                          nidx, noff, wl.batch)
        sc.flush_cache()
        assert sc.sync_status() == 0
        ut = np.searchsorted(rb, ug, side="right") - 1
        for t in range(wl.num_tables):
            sel = ut == t
            rows_t = ug[sel] - rb[t]
            assert_close(tabs[t].np[rows_t], nr[sel].astype(np.float32), f"updated rows of table {t}")
            assert_close(state[t].np[rows_t], ns[sel].astype(np.float32), f"accumulators of table {t}")
        rc, want = oracle.embedding_bag_fwd(wl.rows, ora_tabs, host[e + 1][0], host[e + 1][1], wl.batch)
        assert rc == 0
        out = sc.embedding_bag_fwd(nidx, noff, wl.batch, rms[(e + 1) % 2])
        assert_close(out.cpu().numpy(), want, f"forward pass of batch {e + 1} after the update of batch {e}")
    assert sc.sync_status() == 0
    assert sc.get_counter(binding.COUNTER_AHEAD_USED) - used0 == 2
    sc.set_tuning(binding.TUNE_LOOKAHEAD, 0)


def _full_size_sgd_step(wl, P, tabs=None):
    """One SGD workload at the size bench.py runs it: build_cache over P profile batches, then one batch through
    remap, forward and backward -- integer outputs bit-exact, pooled sums and every updated row within tolerance --
    the backward pass a second time in bench.py's launch configuration (sort started by remap on the side stream)."""
    from gpu_harness import assert_bf16_within
    dev = torch.device("cuda:0")
    bf16 = wl.dtype == "bf16"
    tabs = tabs if tabs is not None else [binding.PinnedArray((wl.rows[t], wl.dim), np.uint16 if bf16 else np.float32)
                                          for t in range(wl.num_tables)]
    for t in range(wl.num_tables):
        p = tabs[t]
        chunk = max(1, (1 << 27) // wl.dim)
        for r0 in range(0, wl.rows[t], chunk):
            r1 = min(wl.rows[t], r0 + chunk)
            v = synth.row_values(wl, t, r0, r1, dev).contiguous()
            p.copy_from_device(v.view(torch.int16) if bf16 else v, r0)
            torch.cuda.synchronize()
    sc = binding.Scars(wl.rows, wl.dim, binding.DTYPE_BF16 if bf16 else binding.DTYPE_F32, [p.ptr for p in tabs],
                       binding.OPT_SGD, None)
    smp = synth.Sampler(wl, dev)
    prof = [smp.batch(p, True) for p in range(P)]
    idx, off = smp.batch(0)
    max_L = max(int(b[0].numel()) for b in prof + [(idx, off)])
    sc.bind_buffers(wl.budget_bytes, max_L, wl.num_bags)
    if wl.bag_lambda is None:      # as bench.py does: one index per bag, so a table gets `batch` lookups (up to 4096
        sc.set_tuning(binding.TUNE_MAX_TABLE_LOOKUPS, wl.batch)   # the backward pass then sorts per table in LDS)
    counts = np.zeros(wl.total_rows, dtype=np.uint32)
    sc.build_cache(None, None, 0, wl.budget_bytes, 0)
    for n, (pi, po) in enumerate(prof):
        rc, counts = oracle.histogram(wl.rows, pi.cpu().numpy(), po.cpu().numpy(), wl.batch, counts)
        assert rc == 0
        sc.build_cache(pi, po, wl.batch, wl.budget_bytes, 1 if n == P - 1 else 2)
    assert sc.sync_status() == 0
    k = oracle.budget_rows(wl.total_rows, wl.row_bytes, wl.budget_bytes)
    assert k == sc.cache_rows()
    _say(wl.name, "oracle hot set over", wl.total_rows, "rows, k =", k)
    rc, hot, slot_of = oracle.hot_set(counts, k)
    assert np.array_equal(sc.counts().cpu().numpy().view(np.uint32), counts)
    assert np.array_equal(sc.hot_gid().cpu().numpy(), hot)
    assert np.array_equal(sc.slot_of().cpu().numpy(), slot_of)
    ora_tabs = [p.np for p in tabs]
    hi, ho = idx.cpu().numpy(), off.cpu().numpy()
    grad = smp.grads(0)
    lr = np.float32(wl.lr)
    _say(wl.name, "oracle step")
    rc, slot, hit, miss, mg = oracle.remap(wl.rows, hi, ho, wl.batch, slot_of)
    rc2, want = oracle.embedding_bag_fwd(wl.rows, ora_tabs, hi, ho, wl.batch)
    rc3, sg, sb, ss, ug = oracle.bwd_segments(wl.rows, hi, ho, wl.batch)
    rc4, nr, ns, gr = oracle.embedding_bag_bwd_update(wl.rows, ora_tabs, None, 0, hi, ho, wl.batch, grad.cpu().numpy(), lr,
                                                      np.float32(0.0), report=True, n_unique=ug.size)
    assert rc == rc2 == rc3 == rc4 == 0
    L = idx.numel()
    # (1) the integer outputs need only the remap and the sort: take them from a backward call with lr = 0, which
    # rewrites every touched row with its own value
    rm = sc.remap(idx, off, wl.batch)
    out = sc.embedding_bag_fwd(idx, off, wl.batch, rm)
    bo = sc.new_bwd_out(L)
    sc.embedding_bag_bwd_update(idx, off, wl.batch, rm, grad, 0.0, 0.0, bo)
    assert sc.sync_status() == 0
    assert rm.n_hit_miss.cpu().tolist() == [hit.size, miss.size] and hit.size + miss.size == L
    assert np.array_equal(rm.slot.cpu().numpy()[:L], slot)
    assert np.array_equal(rm.hit_pos.cpu().numpy()[: hit.size], hit)
    assert np.array_equal(rm.miss_pos.cpu().numpy()[: miss.size], miss)
    assert np.array_equal(rm.miss_gid.cpu().numpy()[: miss.size], mg)
    assert_close(out.cpu().numpy(), want, f"pooled output, {wl.name} at full size")
    U, nv = bo.n_unique.cpu().tolist()
    assert U == ug.size and nv == sg.size
    assert np.array_equal(bo.sorted_gid.cpu().numpy()[:nv], sg)
    assert np.array_equal(bo.sorted_bag.cpu().numpy()[:nv], sb)
    assert np.array_equal(bo.seg_start.cpu().numpy()[: U + 1], ss)
    assert np.array_equal(bo.unique_gid.cpu().numpy()[:U], ug)
    del bo
    # (2) the real step, as bench.py launches it
    sc.set_tuning(binding.TUNE_PRESORT, 131072)
    rm = sc.remap(idx, off, wl.batch, rm)
    sc.embedding_bag_fwd(idx, off, wl.batch, rm, out)
    sc.embedding_bag_bwd_update(idx, off, wl.batch, rm, grad, float(lr), 0.0)
    sc.flush_cache()
    assert sc.sync_status() == 0
    assert sc.get_counter(binding.COUNTER_PREPARED_USED) == (1 if L >= 131072 and k < wl.total_rows else 0)
    rb = wl.row_base
    ut = np.searchsorted(rb, ug, side="right") - 1
    for t in range(wl.num_tables):
        sel = ut == t
        if bf16:
            assert_bf16_within(tabs[t].np[ug[sel] - rb[t]], nr[sel], f"updated bf16 rows of table {t}")
        else:
            assert_close(tabs[t].np[ug[sel] - rb[t]], nr[sel].astype(np.float32), f"updated rows of table {t}")
    # (3) one step in the look-ahead order, as bench.py's second leg runs it: batch 0 once more, batch 1 behind it
    sc.set_tuning(binding.TUNE_LOOKAHEAD, 1)
    nidx, noff = smp.batch(1)
    if int(nidx.numel()) <= max_L:
        rm2 = sc.new_remap_out(max_L)
        sc.remap(idx, off, wl.batch, rm)
        sc.embedding_bag_fwd(idx, off, wl.batch, rm, out)
        rc4, nr, ns, gr = oracle.embedding_bag_bwd_update(wl.rows, ora_tabs, None, 0, hi, ho, wl.batch, grad.cpu().numpy(), lr,
                                                          np.float32(0.0), report=True, n_unique=ug.size)
        assert rc4 == 0
        sc.remap(nidx, noff, wl.batch, rm2)
        sc.embedding_bag_bwd_update_ahead(idx, off, wl.batch, rm, grad, float(lr), 0.0, rm2, nidx, noff, wl.batch)
        sc.flush_cache()
        assert sc.sync_status() == 0
        for t in range(wl.num_tables):
            sel = ut == t
            if bf16:
                assert_bf16_within(tabs[t].np[ug[sel] - rb[t]], nr[sel], f"look-ahead: updated bf16 rows of table {t}")
            else:
                assert_close(tabs[t].np[ug[sel] - rb[t]], nr[sel].astype(np.float32), f"look-ahead: updated rows of table {t}")
        rc5, want2 = oracle.embedding_bag_fwd(wl.rows, ora_tabs, nidx.cpu().numpy(), noff.cpu().numpy(), wl.batch)
        assert rc5 == 0
        out2 = sc.embedding_bag_fwd(nidx, noff, wl.batch, rm2)
        assert_close(out2.cpu().numpy(), want2, f"look-ahead: pooled output of the next batch, {wl.name} at full size")
        assert sc.sync_status() == 0
        assert sc.get_counter(binding.COUNTER_AHEAD_USED) == (1 if k < wl.total_rows else 0)
    sc.close()
    for p in tabs:
        p.free()
    return max_L


@pytest.mark.timeout(900)
def test_full_size_low_skew_bf16_matches_oracle():
    """26 bf16 tables, 50M rows x dim 64, batch 16384, bags 1+Poisson(9), Zipf 0.5, 10 % of rows cached: 4.3M lookups
    per batch, so the sort runs its large tiles and the compactions span more than two thousand tiles."""
    assert _full_size_sgd_step(synth.workload("low_skew"), 4) > (1 << 21)


@pytest.mark.timeout(900)
def test_full_size_dlrm_onehot_matches_oracle():
    """26 fp32 tables of 10 to 10M rows x dim 64, batch 2048, one index per table and sample, Zipf 1.1, 5 % cached."""
    _full_size_sgd_step(synth.workload("dlrm_onehot"), 8)


@pytest.mark.timeout(900)
def test_full_size_low_skew_uniform_bf16_matches_oracle():
    """The uniform variant of the same configuration: hardly any repeated row, so the cache catches only its own
    share of the lookups (10 %) and nearly every sorted run has one lookup."""
    assert _full_size_sgd_step(synth.workload("low_skew_uniform"), 4) > (1 << 21)
