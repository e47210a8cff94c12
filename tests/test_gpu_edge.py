"""Edge cases of the HIP path against the oracle: empty inputs, ties, extreme budgets, long segments,
out-of-range indices, bad offsets."""
import ctypes as C

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import oracle
from paper_2411_01611_amd import binding, synth
from gpu_harness import GpuCase, assert_close


def _say(*a):
    print(*a, flush=True)


def _custom_case(rows, D, idx, off, B, budget_rows, optimizer="sgd", dtype="f32", nprofile=0):
    wl = synth.Workload("custom", tuple(rows), D, dtype, B, None, 1.0, budget_rows * D * (4 if dtype == "f32" else 2),
                        optimizer)
    c = GpuCase(wl, nprofile=nprofile, max_L=max(len(idx), 1))
    c.batch = (torch.tensor(idx, dtype=torch.int32), torch.tensor(off, dtype=torch.int32))
    return c


def _run_all(c, profile_with_batch=True, with_out=True):
    """build (profile = the batch itself), remap, fwd, bwd on both sides; returns GPU outputs (with_out False: the
    backward pass is not asked for its sorted segments, and bo is None)."""
    wl = c.wl
    idx, off = c.batch
    if profile_with_batch:
        c.profile = [c.batch]
    counts, hot, slot_of = c.build()
    d_idx, d_off = c.dev_batch()
    rm = c.s.remap(d_idx, d_off, wl.batch)
    out = c.s.embedding_bag_fwd(d_idx, d_off, wl.batch, rm)
    g = torch.Generator().manual_seed(5)
    grad = torch.randn(wl.num_bags, wl.dim, generator=g)
    bo = c.s.new_bwd_out(max(idx.numel(), 1)) if with_out else None
    c.s.embedding_bag_bwd_update(d_idx, d_off, wl.batch, rm, grad.to(c.dev), 0.01, 1e-8, bo)
    c.s.flush_cache()
    return rm, out, bo, grad


@pytest.mark.parametrize("D,dtype,opt", [(32, "f32", "sgd"), (32, "f32", "adagrad"), (24, "f32", "adagrad"),
                                         (256, "f32", "sgd"), (512, "bf16", "sgd"), (64, "bf16", "adagrad")])
@pytest.mark.parametrize("one_launch", [True, False])
def test_long_segments(D, dtype, opt, one_launch):
    """Rows looked up thousands of times: runs far above the 64-lookup task size, spanning several sort tiles,
    for lane groups narrower than, equal to and wider than a wave, and a row width that is not a power of two."""
    _long_segments_case(D, dtype, opt, one_launch, B=6000, budget_rows=100, table_limit=0)


@pytest.mark.parametrize("D,dtype,opt", [(32, "f32", "sgd"), (24, "f32", "adagrad"), (256, "f32", "sgd"),
                                         (512, "bf16", "sgd"), (64, "bf16", "adagrad")])
@pytest.mark.parametrize("budget_rows", [100, 2, 0])
@pytest.mark.parametrize("with_out", [True, False])
def test_long_runs_when_the_caller_has_stated_the_lookups_per_table(D, dtype, opt, budget_rows, with_out):
    """The same runs under SCARS_TUNE_MAX_TABLE_LOOKUPS: each long run is summed by the workgroup of the chunk it starts
    in (no partial sums, no combining launch), with the long-run rows cached (100), mostly in host memory (2: only
    the two longest are cached) and all in host memory (0).  Asked for the sorted segments the backward pass lists the
    runs (k_small_segments) and updates run by run; not asked, it updates by position (k_small_update)."""
    _long_segments_case(D, dtype, opt, True, B=4000, budget_rows=budget_rows, table_limit=4000, with_out=with_out)


def _long_segments_case(D, dtype, opt, one_launch, B, budget_rows, table_limit, with_out=True):
    rng = np.random.default_rng(3)
    rows = [50, 1000]
    idx0 = np.where(rng.random(B) < 0.7, 7, rng.integers(0, 50, B))        # 70 % of table 0 hits row 7
    idx1 = np.where(rng.random(B) < 0.3, 999, rng.integers(0, 1000, B))    # long run at the very end of key space
    idx1[:130] = 500                                                         # a run of just over two tasks
    idx1[130:195] = 501                                                      # 65 lookups: the shortest long run
    idx1[195:259] = 502                                                      # 64 lookups: the longest short run
    idx = np.concatenate([idx0, idx1]).astype(np.int32)
    off = np.arange(2 * B + 1, dtype=np.int32)
    _say("D", D, dtype, opt, "one launch" if one_launch else "two launches", "B", B, "cached rows", budget_rows,
         "table limit", table_limit)
    c = _custom_case(rows, D, idx, off, B, budget_rows=budget_rows, optimizer=opt, dtype=dtype)
    if not one_launch:      # long runs and the other rows in launches of their own, as large batches do
        c.s.set_tuning(binding.TUNE_FUSED_LONG_MAX_L, 0)
    if table_limit:
        c.s.set_tuning(binding.TUNE_MAX_TABLE_LOOKUPS, table_limit)
        c.s.profile_enable(True)
    rm, out, bo, grad = _run_all(c, with_out=with_out)
    assert c.s.sync_status() == 0
    if table_limit:
        prof = c.s.profile_read()
        c.s.profile_enable(False)
        assert "seg_combine" not in prof, prof
        if with_out:
            assert "small_segments" in prof and "seg_rows_long" in prof and "small_update" not in prof, prof
        else:
            assert "small_update" in prof and "small_segments" not in prof and "seg_rows_long" not in prof, prof
    wl = c.wl
    rc, want = oracle.embedding_bag_fwd(rows, c.ora_tables, idx, off, B)
    assert_close(out.cpu().numpy(), want, "forward")
    rc, sg, sb, ss, ug = oracle.bwd_segments(wl.rows, idx, off, B)
    if with_out:
        assert np.array_equal(bo.sorted_gid.cpu().numpy()[: sg.size], sg)
        assert np.array_equal(bo.sorted_bag.cpu().numpy()[: sb.size], sb)
        assert np.array_equal(bo.seg_start.cpu().numpy()[: ss.size], ss)
    o = 1 if opt == "adagrad" else 0
    rc, nr, ns, gr = oracle.embedding_bag_bwd_update(wl.rows, c.ora_tables, c.ora_state, o, idx, off, B, grad.numpy(),
                                                     np.float32(0.01), np.float32(1e-8), report=True, n_unique=ug.size)
    oracle.embedding_bag_bwd_update(wl.rows, c.ora_tables, c.ora_state, o, idx, off, B, grad.numpy(),
                                    np.float32(0.01), np.float32(1e-8))
    if dtype == "f32":
        assert_close(c.pinned_rows(), np.concatenate(c.ora_tables), "rows with long segments")
    else:
        from gpu_harness import assert_bf16_within
        assert_bf16_within(c.pinned_rows()[ug], nr, "bf16 rows with long segments")
    if opt == "adagrad":
        assert_close(c.pinned_state_rows(), np.concatenate(c.ora_state), "state with long segments")
    c.close()


def test_empty_bags_and_ragged_lengths():
    rng = np.random.default_rng(11)
    rows = [300, 17, 4000]
    B = 513
    lens = rng.integers(0, 5, 3 * B)
    lens[:7] = 0
    lens[-3:] = 0
    lens[100] = 700                                    # one very long bag
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    idx = np.concatenate([rng.integers(0, rows[t], int(lens[t * B:(t + 1) * B].sum())) for t in range(3)]).astype(np.int32)
    c = _custom_case(rows, 8, idx, off, B, budget_rows=400)
    rm, out, bo, grad = _run_all(c)
    assert c.s.sync_status() == 0
    rc, want = oracle.embedding_bag_fwd(rows, [x.copy() for x in c.ora_tables], idx, off, B)
    assert_close(out.cpu().numpy(), want, "ragged bags")
    assert np.all(out.cpu().numpy()[lens == 0] == 0.0)
    rc, sg, sb, ss, ug = oracle.bwd_segments(rows, idx, off, B)
    assert np.array_equal(bo.sorted_bag.cpu().numpy()[: sb.size], sb)
    oracle.embedding_bag_bwd_update(rows, c.ora_tables, None, 0, idx, off, B, grad.numpy(), np.float32(0.01), np.float32(0))
    assert_close(c.pinned_rows(), np.concatenate(c.ora_tables), "rows after ragged update")
    c.close()


def test_empty_batch():
    rows = [10, 10]
    B = 4
    off = np.zeros(2 * B + 1, dtype=np.int32)
    c = _custom_case(rows, 4, [], off, B, budget_rows=5)
    c.profile = []
    c.build()
    d_off = torch.tensor(off, dtype=torch.int32, device=c.dev)
    d_idx = torch.empty(0, dtype=torch.int32, device=c.dev)
    rm = c.s.remap(d_idx, d_off, B)
    assert rm.n_hit_miss.cpu().tolist() == [0, 0]
    out = c.s.embedding_bag_fwd(d_idx, d_off, B, rm)
    assert torch.count_nonzero(out).item() == 0
    bo = c.s.new_bwd_out(1)
    before = c.pinned_rows().copy()
    c.s.embedding_bag_bwd_update(d_idx, d_off, B, rm, torch.ones(2 * B, 4, device=c.dev), 0.1, 0.0, bo)
    c.s.flush_cache()
    assert c.s.sync_status() == 0
    assert bo.n_unique.cpu().tolist() == [0, 0] and int(bo.seg_start[0]) == 0
    assert np.array_equal(c.pinned_rows(), before)
    # all-zero counts: the hot set is the lowest ids
    assert c.s.hot_gid().cpu().tolist() == [0, 1, 2, 3, 4]
    c.close()


def test_tie_classes_and_extreme_budgets():
    rows = [3000, 2500]
    N = sum(rows)
    B = 4096
    rng = np.random.default_rng(2)
    # counts are small integers with huge tie classes; boundary falls inside a class that spans both tables
    idx = np.concatenate([rng.integers(0, 3000, B), rng.integers(0, 2500, B)]).astype(np.int32)
    off = np.arange(2 * B + 1, dtype=np.int32)
    for kb in (0, 1, 2047, 2048, 2049, 4000, N - 1, N, N + 10):
        _say("budget rows", kb)
        c = _custom_case(rows, 4, idx, off, B, budget_rows=kb)
        c.profile = [c.batch]
        counts, hot, slot_of = c.build()
        assert c.s.sync_status() == 0
        assert c.s.cache_rows() == min(kb, N)
        assert np.array_equal(c.s.hot_gid().cpu().numpy(), hot)
        assert np.array_equal(c.s.slot_of().cpu().numpy(), slot_of)
        rm = c.s.remap(*c.dev_batch(), B)
        nh, nm = rm.n_hit_miss.cpu().tolist()
        assert nh + nm == 2 * B
        if kb == 0:
            assert nh == 0          # no cache: every lookup is communicated (the paper's baseline, eq. (4))
        if kb >= N:
            assert nm == 0
        c.close()


def test_large_counts_use_all_select_passes():
    """Counts written directly (profile of zero lookups, accumulate on preset counts) exercise the high digits."""
    rows = [5000]
    c = _custom_case(rows, 4, [0], [0, 1], 1, budget_rows=1234)
    rng = np.random.default_rng(8)
    counts = rng.integers(0, 2 ** 32, 5000, dtype=np.uint64).astype(np.uint32)
    counts[100:200] = counts[100]                       # a tie class among large values
    c.s.build_cache(None, None, 0, c.budget, 0)
    c.s.counts().copy_(torch.from_numpy(counts.view(np.int32)))
    c.s.build_cache(None, None, 0, c.budget, 1)
    rc, hot, slot_of = oracle.hot_set(counts, 1234)
    assert np.array_equal(c.s.hot_gid().cpu().numpy(), hot)
    assert np.array_equal(c.s.slot_of().cpu().numpy(), slot_of)
    c.close()


@pytest.mark.parametrize("small_sort", [False, True, "update by position"])
def test_out_of_range_index_is_latched_and_treated_as_absent(small_sort):
    rows = [40, 30]
    B = 64
    rng = np.random.default_rng(4)
    idx = np.concatenate([rng.integers(0, 40, B), rng.integers(0, 30, B)]).astype(np.int32)
    idx[5] = 40
    idx[70] = -1
    idx[127] = 1000
    off = np.arange(2 * B + 1, dtype=np.int32)
    c = _custom_case(rows, 4, idx, off, B, budget_rows=20)
    if small_sort:     # each table's pairs sorted by a workgroup of their own: invalid lookups still end up last of all
        c.s.set_tuning(binding.TUNE_MAX_TABLE_LOOKUPS, B)
    c.profile = []
    c.build()
    d_idx, d_off = c.dev_batch()
    c.s.build_cache(d_idx, d_off, B, c.budget, 0)
    assert c.s.sync_status() == binding.ERR_INDEX_RANGE
    assert c.s.sync_status() == 0                                   # reading clears the latch
    rc, counts = oracle.histogram(rows, idx, off, B)
    assert rc == oracle.ERR_INDEX_RANGE
    assert np.array_equal(c.s.counts().cpu().numpy().view(np.uint32), counts)
    rc, hot, slot_of = oracle.hot_set(counts, 20)
    assert np.array_equal(c.s.hot_gid().cpu().numpy(), hot)
    rm = c.s.remap(d_idx, d_off, B)
    assert c.s.sync_status() == binding.ERR_INDEX_RANGE
    rc, slot, hit, miss, mg = oracle.remap(rows, idx, off, B, slot_of)
    assert rm.n_hit_miss.cpu().tolist() == [hit.size, miss.size] and hit.size + miss.size == 2 * B - 3
    assert np.array_equal(rm.slot.cpu().numpy(), slot)
    assert np.array_equal(rm.miss_gid.cpu().numpy()[: mg.size], mg)
    out = c.s.embedding_bag_fwd(d_idx, d_off, B, rm)
    rc, want = oracle.embedding_bag_fwd(rows, c.ora_tables, idx, off, B)
    assert rc == oracle.ERR_INDEX_RANGE
    assert_close(out.cpu().numpy(), want, "invalid lookups add nothing")
    grad = torch.ones(2 * B, 4)
    by_position = small_sort == "update by position"    # (not asked for the sorted segments: no list of runs is made)
    bo = None if by_position else c.s.new_bwd_out(2 * B)
    c.s.embedding_bag_bwd_update(d_idx, d_off, B, rm, grad.to(c.dev), 0.5, 0.0, bo)
    c.s.flush_cache()
    c.s.sync_status()
    rc, sg, sb, ss, ug = oracle.bwd_segments(rows, idx, off, B)
    if not by_position:
        assert bo.n_unique.cpu().tolist() == [ug.size, sg.size]
        assert np.array_equal(bo.sorted_gid.cpu().numpy()[: sg.size], sg)
        assert np.array_equal(bo.seg_start.cpu().numpy()[: ss.size], ss)
    oracle.embedding_bag_bwd_update(rows, c.ora_tables, None, 0, idx, off, B, grad.numpy(), np.float32(0.5), np.float32(0))
    assert_close(c.pinned_rows(), np.concatenate(c.ora_tables), "rows after update with invalid lookups")
    c.close()


def test_more_lookups_in_a_table_than_stated_is_latched_and_stays_in_bounds():
    """SCARS_TUNE_MAX_TABLE_LOOKUPS is a statement of the caller's; a batch that breaks it is reported, not trusted."""
    wl = synth.workload("tiny")                                    # 256 lookups per table
    c = GpuCase(wl)
    c.build()
    d_idx, d_off = c.dev_batch()
    grad = c.sampler.grads(0).to(c.dev)
    c.s.set_tuning(binding.TUNE_MAX_TABLE_LOOKUPS, 100)
    rm = c.s.remap(d_idx, d_off, wl.batch)
    assert c.s.sync_status() == 0                                   # remap does not depend on it
    out = c.s.embedding_bag_fwd(d_idx, d_off, wl.batch, rm)
    # the fetch's launch carried the per-table sort, which found the statement broken; the pooled sums are not affected
    assert c.s.sync_status() == binding.ERR_OFFSETS
    rc, want = oracle.embedding_bag_fwd(wl.rows, c.ora_tables, c.batch[0].numpy(), c.batch[1].numpy(), wl.batch)
    assert rc == 0
    assert_close(out.cpu().numpy(), want, "forward pass beside a refused sort")
    c.s.embedding_bag_bwd_update(d_idx, d_off, wl.batch, rm, grad, 0.01, 0.0)      # in bounds, results unspecified
    c.s.sync_status()
    rm = c.s.remap(d_idx, d_off, wl.batch)
    c.s.embedding_bag_bwd_update(d_idx, d_off, wl.batch, rm, grad, 0.01, 0.0)      # this one sorts for itself
    assert c.s.sync_status() == binding.ERR_OFFSETS
    assert c.s.sync_status() == 0
    c.s.set_tuning(binding.TUNE_MAX_TABLE_LOOKUPS, 10 ** 6)         # beyond what the per-table sort takes: the general sort
    bo = c.s.new_bwd_out()
    c.s.embedding_bag_bwd_update(d_idx, d_off, wl.batch, rm, grad, 0.01, 0.0, bo)
    assert c.s.sync_status() == 0
    rc, sg, sb, ss, ug = oracle.bwd_segments(wl.rows, c.batch[0].numpy(), c.batch[1].numpy(), wl.batch)
    assert bo.n_unique.cpu().tolist() == [ug.size, sg.size]
    assert np.array_equal(bo.sorted_gid.cpu().numpy()[: sg.size], sg)
    c.close()


def test_bad_offsets_are_latched():
    rows = [40, 30]
    B = 8
    idx = np.arange(16, dtype=np.int32) % 30
    c = _custom_case(rows, 4, idx, np.arange(17, dtype=np.int32), B, budget_rows=10)
    c.profile = [c.batch]
    c.build()
    assert c.s.sync_status() == 0
    for bad in ([0, 1, 2, 3, 5, 4, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15, 16],      # decreasing
                [1] + list(range(1, 17)),                                           # does not start at 0
                list(range(16)) + [15]):                                            # does not end at L
        d_off = torch.tensor(bad, dtype=torch.int32, device=c.dev)
        d_idx = torch.tensor(idx, dtype=torch.int32, device=c.dev)
        rm = c.s.remap(d_idx, d_off, B)
        c.s.embedding_bag_fwd(d_idx, d_off, B, rm)          # stays in bounds whatever the offsets say
        assert c.s.sync_status() == binding.ERR_OFFSETS
        assert oracle.remap(rows, idx, np.array(bad, dtype=np.int32), B, c.ora_slot_of)[0] == oracle.ERR_OFFSETS
    c.close()


def test_rebuild_after_updates_keeps_updated_rows():
    """A second build_cache writes updated hot rows back before it reselects."""
    wl = synth.workload("tiny")
    c = GpuCase(wl)
    c.build()
    d_idx, d_off = c.dev_batch()
    rm = c.s.remap(d_idx, d_off, wl.batch)
    grad = c.sampler.grads(0)
    c.s.embedding_bag_bwd_update(d_idx, d_off, wl.batch, rm, grad.to(c.dev), 0.01, 0.0)
    oracle.embedding_bag_bwd_update(wl.rows, c.ora_tables, None, 0, c.batch[0].numpy(), c.batch[1].numpy(), wl.batch,
                                    grad.numpy(), np.float32(0.01), np.float32(0))
    c.s.build_cache(None, None, 0, c.budget // 2, 1)            # reselect with half the budget, no flush call
    assert c.s.sync_status() == 0
    assert c.s.cache_rows() == c.k // 2
    rm = c.s.remap(d_idx, d_off, wl.batch)
    out = c.s.embedding_bag_fwd(d_idx, d_off, wl.batch, rm)
    rc, want = oracle.embedding_bag_fwd(wl.rows, c.ora_tables, c.batch[0].numpy(), c.batch[1].numpy(), wl.batch)
    assert_close(out.cpu().numpy(), want, "forward after rebuild")
    c.close()


def test_binding_new_buffers_starts_over_on_the_same_handle():
    """scars_bind_buffers on a handle that has already run steps: the old cache is gone (the caller flushed it), a
    per-batch call before the next build_cache is refused, and with another budget and a larger max_L the path matches
    the oracle again on the rows the first steps left in host memory."""
    wl = synth.workload("multi_hot", scale=0.004, batch=200)
    c = GpuCase(wl)
    c.build()
    s = c.s
    lr, eps = np.float32(wl.lr), np.float32(wl.eps)

    def step(e):
        idx, off = c.sampler.batch(e)
        grad = c.sampler.grads(e)
        d_idx, d_off = idx.to(c.dev), off.to(c.dev)
        rm = s.remap(d_idx, d_off, wl.batch)
        out = s.embedding_bag_fwd(d_idx, d_off, wl.batch, rm)
        rc, want = oracle.embedding_bag_fwd(wl.rows, c.ora_tables, idx.numpy(), off.numpy(), wl.batch)
        assert rc == 0
        assert_close(out.cpu().numpy(), want, f"forward of step {e}")
        s.embedding_bag_bwd_update(d_idx, d_off, wl.batch, rm, grad.to(c.dev), float(lr), float(eps))
        (rc,) = oracle.embedding_bag_bwd_update(wl.rows, c.ora_tables, c.ora_state, 1, idx.numpy(), off.numpy(), wl.batch,
                                                grad.numpy(), lr, eps)
        assert rc == 0

    step(0)
    s.flush_cache()
    assert s.sync_status() == 0
    torch.cuda.synchronize()
    old = s.bufs                                              # keep the old buffers alive until the new ones are bound
    c.budget = wl.budget_bytes * 3
    s.bind_buffers(c.budget, 2 * s.max_L, wl.num_bags)
    del old
    assert s.cache_rows() == -1
    idx, off = c.batch
    with pytest.raises(binding.ScarsError):
        s.remap(idx.to(c.dev), off.to(c.dev), wl.batch)       # nothing selected yet under the new buffers
    counts, hot, slot_of = c.build()
    assert np.array_equal(s.hot_gid().cpu().numpy(), hot)
    assert np.array_equal(s.slot_of().cpu().numpy(), slot_of)
    step(1)
    step(2)
    s.flush_cache()
    assert s.sync_status() == 0
    assert_close(c.pinned_rows(), np.concatenate(c.ora_tables), "rows after binding new buffers")
    assert_close(c.pinned_state_rows(), np.concatenate(c.ora_state), "accumulators after binding new buffers")
    c.close()


def test_two_handles_on_two_streams_do_not_disturb_each_other():
    """Two handles (different tables, row widths and optimizers), each driven on a stream of its own with the
    other's calls issued in between, one of them with its side streams on: each matches the oracle as if alone."""
    wls = [synth.workload("multi_hot", scale=0.004, batch=333), synth.workload("dlrm_onehot", scale=0.004, batch=1500)]
    cs = [GpuCase(w, max_L=2 * 333 * 8 * 20 if i == 0 else 0) for i, w in enumerate(wls)]
    cs[0].s.set_tuning(binding.TUNE_PRESORT, 1)
    for c in cs:
        c.build()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    outs = [[], []]
    for e in range(3):
        staged = []
        for i, c in enumerate(cs):                      # remap + forward of both, then the backward passes of both
            wl = c.wl
            idx, off = c.sampler.batch(e)
            grad = c.sampler.grads(e)
            with torch.cuda.stream(streams[i]):
                d_idx, d_off, d_grad = idx.to(c.dev), off.to(c.dev), grad.to(c.dev)
                rm = c.s.remap(d_idx, d_off, wl.batch)
                out = c.s.embedding_bag_fwd(d_idx, d_off, wl.batch, rm).clone()
            staged.append((idx, off, grad, d_idx, d_off, d_grad, rm, out))
        for i, c in enumerate(cs):
            wl = c.wl
            idx, off, grad, d_idx, d_off, d_grad, rm, out = staged[i]
            with torch.cuda.stream(streams[i]):
                c.s.embedding_bag_bwd_update(d_idx, d_off, wl.batch, rm, d_grad, float(wl.lr), float(wl.eps))
            rc, want = oracle.embedding_bag_fwd(wl.rows, c.ora_tables, idx.numpy(), off.numpy(), wl.batch)
            assert rc == 0
            outs[i].append((out, want))
            (rc,) = oracle.embedding_bag_bwd_update(wl.rows, c.ora_tables, c.ora_state, 1 if wl.optimizer == "adagrad" else 0,
                                                    idx.numpy(), off.numpy(), wl.batch, grad.numpy(), np.float32(wl.lr),
                                                    np.float32(wl.eps))
            assert rc == 0
        for st in streams:
            st.synchronize()                            # the batch tensors above are released only now
    for i, c in enumerate(cs):
        with torch.cuda.stream(streams[i]):
            c.s.flush_cache()
            assert c.s.sync_status() == 0
        for e, (out, want) in enumerate(outs[i]):
            assert_close(out.cpu().numpy(), want, f"handle {i} forward of step {e}")
    assert cs[0].s.get_counter(binding.COUNTER_PREPARED_USED) == 3
    assert_close(cs[0].pinned_rows(), np.concatenate(cs[0].ora_tables), "fp32 rows of the first handle")
    assert_close(cs[0].pinned_state_rows(), np.concatenate(cs[0].ora_state), "accumulators of the first handle")
    assert_close(cs[1].pinned_rows(), np.concatenate(cs[1].ora_tables), "rows of the second handle")
    for c in cs:
        c.close()


def test_backward_never_reads_stale_staged_rows():
    """The backward pass may take cold rows from the staging area filled by the forward pass of the same batch,
    but not after the arrays were reused for another batch, nor after the rows were already updated once."""
    wl = synth.workload("multi_hot", scale=0.004, batch=200)
    c = GpuCase(wl)
    c.build()
    s = c.s
    A, B2 = c.sampler.batch(0), c.sampler.batch(1)
    grad = c.sampler.grads(0)
    lr, eps = np.float32(wl.lr), np.float32(wl.eps)
    rm = s.new_remap_out()
    dA, dB = [t.to(c.dev) for t in A], [t.to(c.dev) for t in B2]

    def ora_step(batch):
        oracle.embedding_bag_bwd_update(wl.rows, c.ora_tables, c.ora_state, 1, batch[0].numpy(), batch[1].numpy(), wl.batch,
                                        grad.numpy(), lr, eps)

    # forward of A, then the same arrays are remapped for B and B is updated: A's staged rows must not be used
    s.remap(dA[0], dA[1], wl.batch, rm)
    s.embedding_bag_fwd(dA[0], dA[1], wl.batch, rm)
    s.remap(dB[0], dB[1], wl.batch, rm)
    s.embedding_bag_bwd_update(dB[0], dB[1], wl.batch, rm, grad.to(c.dev), float(lr), float(eps))
    ora_step(B2)
    # forward + backward of A (staged rows used), then a second backward of A without a new forward
    s.remap(dA[0], dA[1], wl.batch, rm)
    s.embedding_bag_fwd(dA[0], dA[1], wl.batch, rm)
    s.embedding_bag_bwd_update(dA[0], dA[1], wl.batch, rm, grad.to(c.dev), float(lr), float(eps))
    ora_step(A)
    s.embedding_bag_bwd_update(dA[0], dA[1], wl.batch, rm, grad.to(c.dev), float(lr), float(eps))
    ora_step(A)
    s.flush_cache()
    assert s.sync_status() == 0
    assert_close(c.pinned_rows(), np.concatenate(c.ora_tables), "rows after interleaved batches")
    assert_close(c.pinned_state_rows(), np.concatenate(c.ora_state), "state after interleaved batches")
    c.close()


@pytest.mark.parametrize("path", ["general sort", "per-table sort", "update by position"])
@pytest.mark.parametrize("seed", range(16))
def test_random_shapes_match_oracle(seed, path):
    """Random small problems: 1 to 6 tables of 1 to 5000 rows, row widths that are and are not powers of two, both
    storage types and optimizers, bag lengths 0 to 12 (with empty bags and duplicates), budgets from nothing to
    everything.  The whole path against the oracle: integers bit-exact, sums and rows within tolerance.  Each problem
    also with the lookups per table stated (SCARS_TUNE_MAX_TABLE_LOOKUPS: each table sorted by a workgroup of its own),
    asked for the sorted segments (a list of runs is made) and not asked (the update goes by position)."""
    from gpu_harness import assert_bf16_within
    rng = np.random.default_rng(1000 + seed)
    T = int(rng.integers(1, 7))
    rows = [int(rng.choice([1, 2, 3, 17, 256, 1000, 5000])) for _ in range(T)]
    dtype = "bf16" if seed % 4 == 3 else "f32"
    D = int(rng.choice([8, 16, 24, 40, 64, 128] if dtype == "bf16" else [4, 8, 12, 16, 20, 32, 64, 100, 128]))
    opt = "adagrad" if seed % 2 else "sgd"
    B = int(rng.choice([1, 2, 63, 64, 65, 300, 1111]))
    max_len = int(rng.choice([1, 2, 5, 12]))
    lens = rng.integers(0, max_len + 1, T * B) if max_len > 1 else np.ones(T * B, dtype=np.int64)
    off = np.zeros(T * B + 1, dtype=np.int32)
    off[1:] = np.cumsum(lens)
    parts = []
    for t in range(T):
        n = int(off[(t + 1) * B] - off[t * B])
        skew = rng.random(n) < 0.5                               # half the lookups go to a few popular rows
        parts.append(np.where(skew, rng.integers(0, min(rows[t], 3), n), rng.integers(0, rows[t], n)))
    idx = np.concatenate(parts).astype(np.int32) if parts else np.zeros(0, dtype=np.int32)
    N = sum(rows)
    k = int(rng.choice([0, 1, N // 3, N]))
    _say("seed", seed, "T", T, "rows", rows, "D", D, dtype, opt, "B", B, "L", idx.size, "k", k)
    c = _custom_case(rows, D, idx, off, B, budget_rows=k, optimizer=opt, dtype=dtype)
    if seed % 3 == 0:
        c.s.set_tuning(binding.TUNE_FUSED_LONG_MAX_L, 0)
    if seed % 4 == 1:
        c.s.set_tuning(binding.TUNE_PAIRS_IN_REMAP, 0)
    per_table = max(int(off[(t + 1) * B] - off[t * B]) for t in range(T))
    if path != "general sort":
        if per_table > 4096:
            c.close()
            pytest.skip("a table gets more lookups than the per-table sort takes")
        c.s.set_tuning(binding.TUNE_MAX_TABLE_LOOKUPS, max(per_table, 1))
    with_out = path != "update by position"
    rm, out, bo, grad = _run_all(c, with_out=with_out)
    assert c.s.sync_status() == 0
    wl = c.wl
    L = idx.size
    rc, slot, hit, miss, mg = oracle.remap(wl.rows, idx, off, B, c.ora_slot_of)
    assert rc == 0 and rm.n_hit_miss.cpu().tolist() == [hit.size, miss.size]
    assert np.array_equal(rm.slot.cpu().numpy()[:L], slot)
    assert np.array_equal(rm.hit_pos.cpu().numpy()[: hit.size], hit)
    assert np.array_equal(rm.miss_pos.cpu().numpy()[: miss.size], miss)
    assert np.array_equal(rm.miss_gid.cpu().numpy()[: miss.size], mg)
    rc, want = oracle.embedding_bag_fwd(rows, c.ora_tables, idx, off, B)
    assert_close(out.cpu().numpy(), want, "forward")
    rc, sg, sb, ss, ug = oracle.bwd_segments(wl.rows, idx, off, B)
    if with_out:
        U, nv = bo.n_unique.cpu().tolist()
        assert U == ug.size and nv == sg.size
        assert np.array_equal(bo.sorted_gid.cpu().numpy()[:nv], sg)
        assert np.array_equal(bo.sorted_bag.cpu().numpy()[:nv], sb)
        assert np.array_equal(bo.seg_start.cpu().numpy()[: U + 1], ss)
        assert np.array_equal(bo.unique_gid.cpu().numpy()[:U], ug)
    o = 1 if opt == "adagrad" else 0
    rc, nr, ns, gr = oracle.embedding_bag_bwd_update(wl.rows, c.ora_tables, c.ora_state, o, idx, off, B, grad.numpy(),
                                                     np.float32(0.01), np.float32(1e-8), report=True, n_unique=ug.size)
    (rc2,) = oracle.embedding_bag_bwd_update(wl.rows, c.ora_tables, c.ora_state, o, idx, off, B, grad.numpy(),
                                             np.float32(0.01), np.float32(1e-8))
    assert rc == 0 and rc2 == 0
    if dtype == "f32":
        assert_close(c.pinned_rows(), np.concatenate(c.ora_tables), "rows")
    else:
        assert_bf16_within(c.pinned_rows()[ug], nr, "bf16 rows")
    if opt == "adagrad":
        assert_close(c.pinned_state_rows(), np.concatenate(c.ora_state), "accumulators")
    c.close()


def test_one_huge_bag_and_one_row_looked_up_a_hundred_thousand_times():
    """A single bag of 300k lookups beside an empty one (the wave-per-bag kernel loops thousands of times) in which
    one row takes a third of the lookups (a run of ~100k positions: thousands of partial sums to combine)."""
    rng = np.random.default_rng(21)
    rows, B, L = [2000], 2, 300_000
    idx = np.where(rng.random(L) < 0.33, 1234, rng.integers(0, 2000, L)).astype(np.int32)
    off = np.array([0, L, L], dtype=np.int32)
    for opt in ("sgd", "adagrad"):
        _say("huge bag", opt)
        c = _custom_case(rows, 32, idx, off, B, budget_rows=500, optimizer=opt)
        rm, out, bo, grad = _run_all(c)
        assert c.s.sync_status() == 0
        rc, want = oracle.embedding_bag_fwd(rows, c.ora_tables, idx, off, B)
        # 150k terms per lane group added one after the other in fp32 (sums reach several hundred) against an fp64
        # sum: rounding grows with the length of the bag, the 1e-5 bar is for bags of the workloads' lengths
        assert np.allclose(out.cpu().numpy(), want, rtol=1e-3, atol=1e-3)
        assert np.all(out.cpu().numpy()[1] == 0.0)
        rc, sg, sb, ss, ug = oracle.bwd_segments(c.wl.rows, idx, off, B)
        U, nv = bo.n_unique.cpu().tolist()
        assert U == ug.size and nv == L
        assert np.array_equal(bo.seg_start.cpu().numpy()[: U + 1], ss)
        o = 1 if opt == "adagrad" else 0
        (rc,) = oracle.embedding_bag_bwd_update(c.wl.rows, c.ora_tables, c.ora_state, o, idx, off, B, grad.numpy(),
                                                np.float32(0.01), np.float32(1e-8))
        assert rc == 0
        assert_close(c.pinned_rows(), np.concatenate(c.ora_tables), "rows after a huge bag")
        if o:
            assert_close(c.pinned_state_rows(), np.concatenate(c.ora_state), "accumulators after a huge bag")
        c.close()


def test_a_thousand_tables():
    """SCARS_MAX_TABLES tables of one to four rows: table search and per-table descriptors at their limit."""
    rng = np.random.default_rng(22)
    T, B = 1024, 3
    rows = [int(r) for r in rng.integers(1, 5, T)]
    lens = rng.integers(0, 3, T * B)
    off = np.zeros(T * B + 1, dtype=np.int32)
    off[1:] = np.cumsum(lens)
    idx = np.concatenate([rng.integers(0, rows[t], int(off[(t + 1) * B] - off[t * B])) for t in range(T)]).astype(np.int32)
    c = _custom_case(rows, 8, idx, off, B, budget_rows=sum(rows) // 2, optimizer="adagrad")
    rm, out, bo, grad = _run_all(c)
    assert c.s.sync_status() == 0
    rc, slot, hit, miss, mg = oracle.remap(c.wl.rows, idx, off, B, c.ora_slot_of)
    assert rm.n_hit_miss.cpu().tolist() == [hit.size, miss.size]
    assert np.array_equal(rm.slot.cpu().numpy()[: idx.size], slot)
    assert np.array_equal(rm.miss_gid.cpu().numpy()[: miss.size], mg)
    rc, want = oracle.embedding_bag_fwd(rows, c.ora_tables, idx, off, B)
    assert_close(out.cpu().numpy(), want, "forward over 1024 tables")
    (rc,) = oracle.embedding_bag_bwd_update(c.wl.rows, c.ora_tables, c.ora_state, 1, idx, off, B, grad.numpy(),
                                            np.float32(0.01), np.float32(1e-8))
    assert_close(c.pinned_rows(), np.concatenate(c.ora_tables), "rows over 1024 tables")
    assert_close(c.pinned_state_rows(), np.concatenate(c.ora_state), "accumulators over 1024 tables")
    c.close()


def test_call_order_and_size_errors_leave_outputs_alone():
    """Errors the host can see are returned before anything is enqueued: no hot set selected yet, a batch larger than
    the buffers were bound for, a budget above the bound one, null arrays."""
    wl = synth.workload("tiny")
    c = GpuCase(wl)                                   # bound, nothing built
    d_idx, d_off = c.dev_batch()
    L = d_idx.numel()
    rm = c.s.new_remap_out()
    rm.slot.fill_(-77)
    out = torch.full((wl.num_bags, wl.dim), 3.5, device=c.dev)
    grad = c.sampler.grads(0).to(c.dev)

    def code(fn):
        with pytest.raises(binding.ScarsError) as e:
            fn()
        return e.value.code

    assert code(lambda: c.s.remap(d_idx, d_off, wl.batch, rm)) == binding.ERR_NOT_BUILT
    assert code(lambda: c.s.embedding_bag_fwd(d_idx, d_off, wl.batch, rm, out)) == binding.ERR_NOT_BUILT
    assert code(lambda: c.s.embedding_bag_bwd_update(d_idx, d_off, wl.batch, rm, grad, 0.01)) == binding.ERR_NOT_BUILT
    assert code(lambda: c.s.flush_cache()) == binding.ERR_NOT_BUILT
    assert code(lambda: c.s.build_cache(d_idx, d_off, wl.batch, c.budget * 2, 0)) == binding.ERR_WORKSPACE
    c.build()
    big_idx = torch.cat([d_idx] * 40)                 # far more lookups than max_L
    big_off = torch.arange(0, wl.num_bags + 1, dtype=torch.int32, device=c.dev) * 40
    assert code(lambda: c.s.remap(big_idx, big_off, wl.batch, rm)) == binding.ERR_WORKSPACE
    assert code(lambda: c.s.remap(d_idx, d_off, wl.batch * 1000, rm)) == binding.ERR_WORKSPACE   # more bags than max_G
    Lb = binding.lib()
    assert Lb.scars_remap(c.s._h, d_idx.data_ptr(), d_off.data_ptr(), L, wl.batch, None, None) == binding.ERR_INVALID_ARG
    assert Lb.scars_remap(c.s._h, None, d_off.data_ptr(), L, wl.batch, C.byref(rm.c()), None) == binding.ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert c.s.sync_status() == 0
    assert bool((rm.slot == -77).all()) and bool((out == 3.5).all())      # nothing was written
    # and the same arrays work once the call is valid
    c.s.remap(d_idx, d_off, wl.batch, rm)
    c.s.embedding_bag_fwd(d_idx, d_off, wl.batch, rm, out)
    rc, want = oracle.embedding_bag_fwd(wl.rows, c.ora_tables, c.batch[0].numpy(), c.batch[1].numpy(), wl.batch)
    assert_close(out.cpu().numpy(), want, "forward after the refused calls")
    c.close()


@pytest.mark.parametrize("n_rows", [1, 2, 5])
def test_tables_of_a_few_rows_sort_with_a_handful_of_bins(n_rows):
    """One table of 1, 2 or 5 rows looked up thousands of times: the radix sort of the backward pass then runs a
    single pass of 1 to 3 bits (2 to 8 bins, fewer than its scan kernel's digit group), over several tiles."""
    rng = np.random.default_rng(n_rows)
    B, per = 700, 5
    L = B * per
    idx = rng.integers(0, n_rows, L).astype(np.int32)
    off = (np.arange(B + 1) * per).astype(np.int32)
    for k in (0, n_rows):
        _say("rows", n_rows, "cached", k)
        c = _custom_case([n_rows], 16, idx, off, B, budget_rows=k, optimizer="adagrad")
        rm, out, bo, grad = _run_all(c)
        assert c.s.sync_status() == 0
        rc, sg, sb, ss, ug = oracle.bwd_segments(c.wl.rows, idx, off, B)
        U, nv = bo.n_unique.cpu().tolist()
        assert rc == 0 and U == ug.size and nv == sg.size == L
        assert np.array_equal(bo.sorted_gid.cpu().numpy()[:nv], sg)
        assert np.array_equal(bo.sorted_bag.cpu().numpy()[:nv], sb)
        assert np.array_equal(bo.seg_start.cpu().numpy()[: U + 1], ss)
        (rc,) = oracle.embedding_bag_bwd_update(c.wl.rows, c.ora_tables, c.ora_state, 1, idx, off, B, grad.numpy(),
                                                np.float32(0.01), np.float32(1e-8))
        assert rc == 0
        assert_close(c.pinned_rows(), np.concatenate(c.ora_tables), "rows")
        assert_close(c.pinned_state_rows(), np.concatenate(c.ora_state), "accumulators")
        c.close()


def test_a_bag_longer_than_the_place_field_of_a_pair_can_count():
    """A pair's value holds the bag and the lookup's place inside it; with 2^17 bags the place saturates at 32767.
    One bag of 40000 lookups over cold rows, some of them first seen beyond that place: their runs must still find
    the rows (from host memory instead of the staged copy) and every row must end up as the oracle's."""
    rng = np.random.default_rng(3)
    B, long_bag, n_long = 1 << 17, 77, 40000
    lens = (rng.random(B) < 0.5).astype(np.int64)
    lens[long_bag] = n_long
    off = np.zeros(B + 1, dtype=np.int32)
    off[1:] = np.cumsum(lens)
    L = int(off[-1])
    n_rows = 60000
    idx = rng.integers(0, 30000, L).astype(np.int32)
    a = int(off[long_bag])
    # the tail of the long bag looks up rows no other lookup touches: their runs start beyond the saturated place
    idx[a + 33000:a + n_long] = 30000 + rng.integers(0, 30000, n_long - 33000)
    for k in (0, 2000):
        _say("long bag, cached rows", k)
        c = _custom_case([n_rows], 8, idx, off, B, budget_rows=k)
        rm, out, bo, grad = _run_all(c)
        assert c.s.sync_status() == 0
        rc, want = oracle.embedding_bag_fwd(c.wl.rows, c.ora_tables, idx, off, B)
        got = out.cpu().numpy()
        others = np.arange(B) != long_bag
        assert_close(got[others], want[others], "forward, the ordinary bags")
        # 40000 terms added in fp32 against an fp64 sum: the 1e-5 bar is for bags of the workloads' lengths
        assert np.allclose(got[long_bag], want[long_bag], rtol=1e-3, atol=1e-4)
        rc, sg, sb, ss, ug = oracle.bwd_segments(c.wl.rows, idx, off, B)
        U, nv = bo.n_unique.cpu().tolist()
        assert U == ug.size and nv == L
        assert np.array_equal(bo.sorted_bag.cpu().numpy()[:nv], sb)
        assert np.array_equal(bo.seg_start.cpu().numpy()[: U + 1], ss)
        (rc,) = oracle.embedding_bag_bwd_update(c.wl.rows, c.ora_tables, None, 0, idx, off, B, grad.numpy(),
                                                np.float32(0.01), np.float32(0.0))
        assert rc == 0
        assert_close(c.pinned_rows(), np.concatenate(c.ora_tables), "rows")
        c.close()
