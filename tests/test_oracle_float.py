"""Pins for the oracle's floating-point steps: pooled forward sum, aggregated backward + optimizer step.

Pins: torch's CPU embedding_bag / autograd / optimizers (library special cases), numpy dense brute force,
pure-gather special case, linearity, mass conservation, source invariance, untouched rows.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from paper_2411_01611_amd import synth
from util import bag_of, gids_of, np_tables

CASES = (("tiny", {}), ("multi_hot", {"scale": 0.004}), ("dlrm_onehot", {"scale": 0.002}))


def _setup(name, kw):
    wl = synth.workload(name, **kw)
    s = synth.Sampler(wl)
    tables = synth.make_tables_cpu(wl)
    idx, off = s.batch(0)
    return wl, s, tables, idx, off


def _torch_fwd(wl, tables, idx, off):
    outs = []
    B = wl.batch
    for t in range(wl.num_tables):
        a = int(off[t * B])
        o = off[t * B:(t + 1) * B].long() - a
        ii = idx[a:int(off[(t + 1) * B])].long()
        outs.append(F.embedding_bag(ii, tables[t].double(), o, mode="sum"))
    return torch.cat(outs)


@pytest.mark.parametrize("name,kw", CASES)
def test_fwd_matches_torch_embedding_bag(ora, name, kw):
    wl, s, tables, idx, off = _setup(name, kw)
    rc, out = ora.embedding_bag_fwd(wl.rows, np_tables(wl, tables), idx.numpy(), off.numpy(), wl.batch)
    assert rc == 0 and out.dtype == np.float32
    ref = _torch_fwd(wl, tables, idx, off).float().numpy()
    np.testing.assert_allclose(out, ref, rtol=1e-6, atol=1e-9)


def test_fwd_onehot_is_a_pure_gather(ora):
    wl, s, tables, idx, off = _setup("tiny", {})
    rc, out = ora.embedding_bag_fwd(wl.rows, np_tables(wl, tables), idx.numpy(), off.numpy(), wl.batch)
    B = wl.batch
    for t in range(wl.num_tables):
        assert np.array_equal(out[t * B:(t + 1) * B], tables[t].numpy()[idx[t * B:(t + 1) * B].numpy()])


def test_fwd_empty_bags_are_zero(ora):
    rows = [3, 2]
    tabs = [np.arange(6, dtype=np.float32).reshape(3, 2) + 1, np.arange(4, dtype=np.float32).reshape(2, 2) + 10]
    off = np.array([0, 0, 2, 2, 3], dtype=np.int32)
    idx = np.array([2, 0, 1], dtype=np.int32)
    rc, out = ora.embedding_bag_fwd(rows, tabs, idx, off, 2)
    assert rc == 0
    assert out.tolist() == [[0, 0], [5 + 1, 6 + 2], [0, 0], [12, 13]]


def test_fwd_linearity(ora):
    wl, s, tables, idx, off = _setup("multi_hot", {"scale": 0.004})
    t2 = [torch.randn_like(t) for t in tables]
    tsum = [(a.double() + b.double()).float() for a, b in zip(tables, t2)]
    f = lambda tt: ora.embedding_bag_fwd(wl.rows, [x.numpy() for x in tt], idx.numpy(), off.numpy(), wl.batch)[1]
    np.testing.assert_allclose(f(tsum), f(tables).astype(np.float64) + f(t2), rtol=2e-6, atol=1e-6)


def test_fwd_source_invariance_cache_vs_table(ora):
    wl, s, tables, idx, off = _setup("multi_hot", {"scale": 0.004})
    nt = np_tables(wl, tables)
    rc, counts = ora.histogram(wl.rows, idx.numpy(), off.numpy(), wl.batch)
    k = wl.total_rows // 20
    rc, hot, slot_of = ora.hot_set(counts, k)
    allrows = np.concatenate(nt)
    cache = np.ascontiguousarray(allrows[hot])
    rc, a = ora.embedding_bag_fwd(wl.rows, nt, idx.numpy(), off.numpy(), wl.batch)
    rc, b = ora.embedding_bag_fwd(wl.rows, nt, idx.numpy(), off.numpy(), wl.batch, slot_of, cache)
    assert rc == 0 and np.array_equal(a, b)
    # and the cache is really what is read: poison it, hits change, pure-miss bags do not
    cache2 = cache + 1.0
    rc, c = ora.embedding_bag_fwd(wl.rows, nt, idx.numpy(), off.numpy(), wl.batch, slot_of, cache2)
    gid = gids_of(wl, idx.numpy(), off.numpy())
    hits_per_bag = np.bincount(bag_of(off.numpy(), gid.shape[0]), weights=(slot_of[gid] >= 0), minlength=wl.num_bags)
    np.testing.assert_allclose(c - a, np.repeat(hits_per_bag[:, None], wl.dim, 1), rtol=0, atol=1e-5)


def test_fwd_bf16_rows(ora):
    wl, s, tables, idx, off = _setup("low_skew", {"scale": 0.0005})
    assert tables[0].dtype == torch.bfloat16
    rc, out = ora.embedding_bag_fwd(wl.rows, np_tables(wl, tables), idx.numpy(), off.numpy(), wl.batch)
    ref = _torch_fwd(wl, tables, idx, off).float().numpy()
    np.testing.assert_allclose(out, ref, rtol=1e-6, atol=1e-9)


# ------------------------------------------------------------------ backward
def _torch_step(wl, tables, idx, off, grad, opt_name, lr, eps, state=None):
    """Dense autograd gradient of sum(out * grad) and one step of torch's own optimizer, in fp64."""
    B = wl.batch
    new_w, new_s = [], []
    for t in range(wl.num_tables):
        w = tables[t].double().clone().requires_grad_(True)
        a = int(off[t * B])
        o = off[t * B:(t + 1) * B].long() - a
        ii = idx[a:int(off[(t + 1) * B])].long()
        out = F.embedding_bag(ii, w, o, mode="sum")
        (out * grad[t * B:(t + 1) * B].double()).sum().backward()
        if opt_name == "sgd":
            opt = torch.optim.SGD([w], lr=lr)
        else:
            opt = torch.optim.Adagrad([w], lr=lr, eps=eps, initial_accumulator_value=0.0)
            if state is not None:
                opt.state[w]["sum"] = state[t].double().clone()
                opt.state[w]["step"] = torch.tensor(0.0)
        opt.step()
        new_w.append(w.detach())
        if opt_name == "adagrad":
            new_s.append(opt.state[w]["sum"].clone())
    return new_w, new_s


@pytest.mark.parametrize("name,kw", CASES)
@pytest.mark.parametrize("opt", ["sgd", "adagrad"])
def test_bwd_matches_torch_autograd_and_optimizer(ora, name, kw, opt):
    wl, s, tables, idx, off = _setup(name, kw)
    grad = s.grads(0)
    lr, eps = np.float32(0.01), np.float32(1e-8)
    state = [torch.rand(t.shape) * 0.5 for t in tables] if opt == "adagrad" else None
    ref_w, ref_s = _torch_step(wl, tables, idx, off, grad, opt, float(lr), float(eps), state)
    mine = [t.clone() for t in tables]
    st = [x.clone() for x in state] if state else None
    (rc,) = ora.embedding_bag_bwd_update(wl.rows, [m.numpy() for m in mine], [x.numpy() for x in st] if st else None,
                                         0 if opt == "sgd" else 1, idx.numpy(), off.numpy(), wl.batch,
                                         grad.numpy(), lr, eps)
    assert rc == 0
    for t in range(wl.num_tables):
        np.testing.assert_allclose(mine[t].numpy(), ref_w[t].float().numpy(), rtol=1e-6, atol=1e-9)
        if opt == "adagrad":
            np.testing.assert_allclose(st[t].numpy(), ref_s[t].float().numpy(), rtol=1e-6, atol=1e-12)
    # untouched rows are bit-identical
    gid = gids_of(wl, idx.numpy(), off.numpy())
    touched = np.zeros(wl.total_rows, dtype=bool); touched[gid] = True
    before = torch.cat(tables).numpy(); after = torch.cat(mine).numpy()
    assert np.array_equal(before[~touched], after[~touched])
    assert not np.array_equal(before[touched], after[touched])


def test_bwd_dense_brute_force_sgd(ora):
    wl, s, tables, idx, off = _setup("tiny", {})
    grad = s.grads(0).numpy()
    gid = gids_of(wl, idx.numpy(), off.numpy())
    dW = np.zeros((wl.total_rows, wl.dim), dtype=np.float64)
    np.add.at(dW, gid, grad[bag_of(off.numpy(), gid.shape[0])].astype(np.float64))
    W = torch.cat(tables).numpy().astype(np.float64)
    ref = (W - float(np.float32(0.01)) * dW).astype(np.float32)
    mine = [t.clone() for t in tables]
    ora.embedding_bag_bwd_update(wl.rows, [m.numpy() for m in mine], None, 0, idx.numpy(), off.numpy(), wl.batch,
                                 grad, 0.01, 0.0)
    assert np.array_equal(torch.cat(mine).numpy(), ref)


def test_bwd_report_mode_and_mass_conservation(ora):
    wl, s, tables, idx, off = _setup("multi_hot", {"scale": 0.004})
    grad = s.grads(0).numpy()
    nt = [t.clone().numpy() for t in tables]
    st = [np.zeros_like(x) for x in nt]
    rc, sg, sb, ss, ug = ora.bwd_segments(wl.rows, idx.numpy(), off.numpy(), wl.batch)
    keep = [x.copy() for x in nt]
    rc, nr, ns, gr = ora.embedding_bag_bwd_update(wl.rows, nt, st, 1, idx.numpy(), off.numpy(), wl.batch, grad,
                                                  0.01, 1e-8, report=True, n_unique=ug.size)
    assert rc == 0 and all(np.array_equal(a, b) for a, b in zip(nt, keep))       # report mode mutates nothing
    lens = np.diff(off.numpy()).astype(np.float64)
    np.testing.assert_allclose(gr.sum(0), (lens[:, None] * grad.astype(np.float64)).sum(0), rtol=1e-9, atol=1e-9)
    ora.embedding_bag_bwd_update(wl.rows, nt, st, 1, idx.numpy(), off.numpy(), wl.batch, grad, 0.01, 1e-8)
    assert np.array_equal(np.concatenate(nt)[ug], nr.astype(np.float32))
    assert np.array_equal(np.concatenate(st)[ug], ns.astype(np.float32))


def test_bwd_bf16_rows_round_to_nearest_even(ora):
    wl, s, tables, idx, off = _setup("low_skew", {"scale": 0.0005})
    grad = s.grads(0)
    nt = [x.copy() for x in np_tables(wl, tables)]
    rc, sg, sb, ss, ug = ora.bwd_segments(wl.rows, idx.numpy(), off.numpy(), wl.batch)
    rc, nr, _, _ = ora.embedding_bag_bwd_update(wl.rows, nt, None, 0, idx.numpy(), off.numpy(), wl.batch,
                                                grad.numpy(), 0.01, 0.0, report=True, n_unique=ug.size)
    ora.embedding_bag_bwd_update(wl.rows, nt, None, 0, idx.numpy(), off.numpy(), wl.batch, grad.numpy(), 0.01, 0.0)
    got = np.concatenate(nt)[ug]
    want = torch.from_numpy(nr.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, want)                      # torch's fp32->bf16 cast is round-to-nearest-even
    ref_w, _ = _torch_step(wl, tables, idx, off, grad, "sgd", float(np.float32(0.01)), 0.0)
    np.testing.assert_allclose(nr, torch.cat(ref_w).numpy()[ug], rtol=1e-12, atol=1e-15)


@pytest.mark.parametrize("seed", range(12))
def test_random_shapes_against_numpy_brute_force(ora, seed):
    """Random small problems (1-6 tables of 1-5000 rows, widths that are not powers of two, empty bags, duplicates,
    both optimizers): every oracle step against its definition written with numpy on global row ids."""
    rng = np.random.default_rng(500 + seed)
    T = int(rng.integers(1, 7))
    rows = [int(rng.choice([1, 2, 3, 17, 256, 1000, 5000])) for _ in range(T)]
    D = int(rng.choice([4, 8, 12, 20, 32, 100]))
    B = int(rng.choice([1, 2, 63, 65, 300]))
    lens = rng.integers(0, 7, T * B)
    off = np.zeros(T * B + 1, dtype=np.int32)
    off[1:] = np.cumsum(lens)
    idx = np.concatenate([rng.integers(0, min(rows[t], 4) if rng.random() < 0.5 else rows[t],
                                       int(off[(t + 1) * B] - off[t * B])) for t in range(T)]).astype(np.int32)
    L, N = idx.size, sum(rows)
    rb = np.concatenate([[0], np.cumsum(rows)])
    bag = np.repeat(np.arange(T * B), lens)
    gid = (rb[bag // B] + idx).astype(np.int64)
    tables = [rng.uniform(-1, 1, (r, D)).astype(np.float32) for r in rows]
    W = np.concatenate(tables).astype(np.float64)
    # histogram and hot set
    rc, counts = ora.histogram(rows, idx, off, B)
    assert rc == 0 and np.array_equal(counts, np.bincount(gid, minlength=N).astype(np.uint32))
    k = int(rng.integers(0, N + 1))
    rc, hot, slot_of = ora.hot_set(counts, k)
    order = np.lexsort((np.arange(N), -counts.astype(np.int64)))[:k]
    assert rc == 0 and np.array_equal(hot, order)
    inv = np.full(N, -1, dtype=np.int32)
    inv[order] = np.arange(k, dtype=np.int32)
    assert np.array_equal(slot_of, inv)
    # remap
    rc, slot, hit, miss, mg = ora.remap(rows, idx, off, B, slot_of)
    assert rc == 0 and np.array_equal(slot, inv[gid])
    assert np.array_equal(hit, np.nonzero(inv[gid] >= 0)[0]) and np.array_equal(miss, np.nonzero(inv[gid] < 0)[0])
    assert np.array_equal(mg, gid[miss])
    # forward
    want = np.zeros((T * B, D), dtype=np.float64)
    np.add.at(want, bag, W[gid])
    rc, out = ora.embedding_bag_fwd(rows, tables, idx, off, B)
    assert rc == 0 and np.allclose(out, want.astype(np.float32), rtol=1e-6, atol=1e-7)
    # segments
    rc, sg, sb, ss, ug = ora.bwd_segments(rows, idx, off, B)
    o = np.argsort(gid, kind="stable")
    assert np.array_equal(sg, gid[o]) and np.array_equal(sb, bag[o])
    assert np.array_equal(ug, np.unique(gid)) and np.array_equal(ss[:-1], np.searchsorted(gid[o], ug)) and ss[-1] == L
    # backward, both optimizers
    grad = rng.standard_normal((T * B, D)).astype(np.float32)
    dW = np.zeros((N, D), dtype=np.float64)
    np.add.at(dW, gid, grad[bag].astype(np.float64))
    lr, eps = np.float32(0.05), np.float32(1e-8)
    mine = [t.copy() for t in tables]
    (rc,) = ora.embedding_bag_bwd_update(rows, mine, None, 0, idx, off, B, grad, lr, np.float32(0.0))
    assert rc == 0 and np.array_equal(np.concatenate(mine), (W - float(lr) * dW).astype(np.float32))
    mine = [t.copy() for t in tables]
    G0 = rng.uniform(0, 2, (N, D)).astype(np.float32)
    st = [G0[rb[t]:rb[t + 1]].copy() for t in range(T)]
    (rc,) = ora.embedding_bag_bwd_update(rows, mine, st, 1, idx, off, B, grad, lr, eps)
    Gn = G0.astype(np.float64) + dW * dW
    touched = np.zeros(N, dtype=bool)
    touched[gid] = True
    Wn = np.where(touched[:, None], W - float(lr) * dW / (np.sqrt(Gn) + float(eps)), W)
    assert rc == 0 and np.array_equal(np.concatenate(st), np.where(touched[:, None], Gn, G0).astype(np.float32))
    assert np.allclose(np.concatenate(mine), Wn.astype(np.float32), rtol=1e-7, atol=1e-8)
