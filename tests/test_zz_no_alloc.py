"""scars_remap_static (the remap whose scratch is the library's static device array, for callers that cannot allocate)
against scars_remap, through the C ABI: two calls in a row, the second on a smaller batch, every output bit for bit.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import oracle
from paper_2411_01611_amd import binding, synth
from gpu_harness import GpuCase


def _say(*a):
    print(*a, flush=True)


def _first_samples(wl, idx, off, n):
    """The sub-batch of the first n samples of every table (table-major jagged layout kept)."""
    B, T = wl.batch, wl.num_tables
    off = off.numpy().astype(np.int64)
    idx = idx.numpy()
    parts, lens = [], []
    for t in range(T):
        a, b = off[t * B], off[t * B + n]
        parts.append(idx[a:b])
        lens.append(np.diff(off[t * B: t * B + n + 1]))
    new_off = np.concatenate([[0], np.cumsum(np.concatenate(lens))]).astype(np.int32)
    return torch.from_numpy(np.concatenate(parts).astype(np.int32)), torch.from_numpy(new_off)


def _same(a: binding.RemapOut, b: binding.RemapOut, L: int):
    na, nb = a.n_hit_miss.cpu().tolist(), b.n_hit_miss.cpu().tolist()
    assert na == nb and na[0] + na[1] == L
    for name in ("slot", "gid", "loc"):
        assert torch.equal(getattr(a, name)[:L], getattr(b, name)[:L]), name
    assert torch.equal(a.hit_pos[: na[0]], b.hit_pos[: na[0]])
    assert torch.equal(a.miss_pos[: na[1]], b.miss_pos[: na[1]])
    assert torch.equal(a.miss_gid[: na[1]], b.miss_gid[: na[1]])
    return na


@pytest.mark.parametrize("name,kw,scan", [("multi_hot", {"scale": 0.004, "batch": 333}, False),
                                          ("multi_hot", {"scale": 0.004, "batch": 333}, True),
                                          ("host_spill", {"scale": 0.0005, "batch": 3000}, False)])
def test_remap_static_matches_remap(name, kw, scan):
    _say("case", name, kw, "scan" if scan else "fused")
    wl = synth.workload(name, **kw)
    c = GpuCase(wl)
    try:
        c.build()
        if scan:
            c.s.set_tuning(binding.TUNE_FUSED_SCAN_MAX_TILES, 0)
        idx, off = c.batch
        small = wl.batch // 3
        for n, (i, o) in ((wl.batch, (idx, off)), (small, _first_samples(wl, idx, off, small))):
            _say("  call with", n, "samples per table,", i.numel(), "lookups")
            L = int(i.numel())
            d_i, d_o = i.to(c.dev), o.to(c.dev)
            want = c.s.remap(d_i, d_o, n)
            got = c.s.new_remap_out(L)
            for t in (got.slot, got.gid, got.loc, got.hit_pos, got.miss_pos, got.miss_gid, got.n_hit_miss):
                t.fill_(-7)
            c.s.remap_static(d_i, d_o, n, got)
            assert c.s.sync_status() == 0
            nhm = _same(got, want, L)
            # ... and against the oracle
            rc, slot, hit, miss, mg = oracle.remap(wl.rows, i.numpy(), o.numpy(), n, c.ora_slot_of)
            assert rc == 0 and nhm == [hit.size, miss.size]
            assert np.array_equal(got.slot.cpu().numpy()[:L], slot)
            assert np.array_equal(got.miss_gid.cpu().numpy()[: miss.size], mg)
            # the forward pass accepts these outputs like those of scars_remap
            out_a = c.s.embedding_bag_fwd(d_i, d_o, n, want)
            out_b = c.s.embedding_bag_fwd(d_i, d_o, n, got)
            assert torch.equal(out_a, out_b)
    finally:
        c.close()


def test_remap_static_limits_and_errors():
    _say("case tiny: limits and the latched error")
    wl = synth.workload("tiny")
    c = GpuCase(wl)
    try:
        c.build()
        d_i, d_o = c.dev_batch()
        L = int(d_i.numel())
        with pytest.raises(binding.ScarsError) as ei:
            c.s.remap_static(d_i, d_o, wl.batch, c.s.new_remap_out(L, coalesce=True))
        assert ei.value.code == binding.ERR_INVALID_ARG
        bad = d_i.clone()
        bad[5] = wl.rows[0] + 3                       # out of range for table 0
        got = c.s.remap_static(bad, d_o, wl.batch, c.s.new_remap_out(L))
        assert c.s.sync_status() == binding.ERR_INDEX_RANGE
        assert c.s.sync_status() == 0                 # cleared
        assert int(got.slot[5]) == -1 and int(got.gid[5]) == -1 and int(got.loc[5]) == -1
        # a clean call afterwards is clean
        got = c.s.remap_static(d_i, d_o, wl.batch, c.s.new_remap_out(L))
        assert c.s.sync_status() == 0
        want = c.s.remap(d_i, d_o, wl.batch)
        _same(got, want, L)
    finally:
        c.close()
