"""The input generators: counter-based RNG, permutation, distributions, batch layout."""
import math

import numpy as np
import pytest
import torch

from paper_2411_01611_amd import synth


def test_mix64_matches_integer_form():
    xs = [0, 1, 2, 12345, (1 << 63) - 1, (1 << 63), (1 << 64) - 1, 0x9E3779B97F4A7C15]
    t = torch.tensor([synth._signed(x) for x in xs], dtype=torch.int64)
    got = [int(v) & ((1 << 64) - 1) for v in synth.mix64(t).tolist()]
    assert got == [synth.mix64_int(x) for x in xs]


def test_uniform_range_and_moments():
    u = synth.uniform01(synth.stream_key(1, 2, 3), torch.arange(200_000))
    assert float(u.min()) >= 0.0 and float(u.max()) < 1.0
    assert abs(float(u.mean()) - 0.5) < 0.005
    assert abs(float(u.var()) - 1.0 / 12.0) < 0.002
    # distinct streams are decorrelated
    v = synth.uniform01(synth.stream_key(1, 2, 4), torch.arange(200_000))
    assert abs(float(((u - 0.5) * (v - 0.5)).mean())) < 0.001


def test_permutation_is_bijection_and_seeded():
    wl = synth.workload("tiny")
    s = synth.Sampler(wl)
    p = s.permutation(1).numpy()
    assert np.array_equal(np.sort(p), np.arange(wl.rows[1]))
    assert not np.array_equal(p, np.arange(wl.rows[1]))
    assert np.array_equal(p, synth.Sampler(wl).permutation(1).numpy())
    assert not np.array_equal(p, s.permutation(2).numpy())


def test_workload_shapes():
    for name in synth.WORKLOAD_NAMES:
        wl = synth.workload(name)
        assert all(r >= 1 for r in wl.rows) and wl.row_bytes % 16 == 0
    assert synth.workload("host_spill").total_rows == 200_000_000
    assert synth.workload("low_skew").total_rows == 50_000_000
    assert max(synth.workload("host_spill").rows) <= 40_000_000
    wl = synth.workload("dlrm_onehot")
    assert wl.num_tables == 26 and min(wl.rows) >= 10 and max(wl.rows) <= 10_000_000
    assert synth.workload("multi_hot").budget_bytes // 512 == 3_906_250


def test_batch_layout_onehot_and_multihot():
    wl = synth.workload("tiny")
    idx, off = synth.Sampler(wl).batch(0)
    assert off.dtype == torch.int32 and idx.dtype == torch.int32
    assert off.tolist() == list(range(wl.num_bags + 1))
    assert int(idx.min()) >= 0 and int(idx.max()) < 10_000
    wl = synth.workload("multi_hot", scale=0.01)
    s = synth.Sampler(wl)
    idx, off = s.batch(3)
    lens = np.diff(off.numpy())
    assert off[0] == 0 and off[-1] == idx.numel() and lens.min() >= 1
    idx2, off2 = s.batch(3)
    assert torch.equal(idx, idx2) and torch.equal(off, off2)
    idx3, _ = s.batch(3, profile=True)
    assert not torch.equal(idx[:100], idx3[:100])


def test_bag_lengths_poisson_mean():
    wl = synth.workload("multi_hot", scale=0.25)
    ln = synth.Sampler(wl).lengths(0, 0, False).double()
    assert abs(float(ln.mean()) - 20.0) < 0.5          # 1 + Poisson(19)
    assert abs(float(ln.var()) - 19.0) < 2.5


def test_zipf_frequencies_follow_probs():
    wl = synth.workload("tiny", batch=200_000)
    s = synth.Sampler(wl)
    idx, off = s.batch(0)
    t = 2
    a, b = int(off[t * wl.batch]), int(off[(t + 1) * wl.batch])
    cnt = np.bincount(idx[a:b].numpy(), minlength=wl.rows[t]).astype(np.float64)
    p = s.row_probs(t).numpy()
    assert abs(p.sum() - 1.0) < 1e-12
    top = np.argsort(-p)[:20]
    n = b - a
    for e in top:
        sd = math.sqrt(n * p[e] * (1 - p[e]))
        assert abs(cnt[e] - n * p[e]) < 5 * sd
    # top-ranked row carries p(1) = 1/H
    assert abs(p.max() - 1.0 / np.sum(np.arange(1, 10_001, dtype=np.float64) ** -1.05)) < 1e-12


def test_rows_and_grads():
    wl = synth.workload("tiny")
    w = synth.make_tables_cpu(wl)
    assert w[0].shape == (10_000, 16) and w[0].dtype == torch.float32
    allw = torch.cat(w)
    assert float(allw.min()) >= -0.01 and float(allw.max()) <= 0.01
    assert abs(float(allw.mean())) < 1e-4
    assert torch.equal(synth.row_values(wl, 1, 5, 9), w[1][5:9])
    g = synth.Sampler(wl).grads(0)
    assert g.shape == (wl.num_bags, 16)
    assert abs(float(g.mean())) < 0.03 and abs(float(g.std()) - 1.0) < 0.03
    wb = synth.make_tables_cpu(synth.workload("low_skew", scale=0.001))
    assert wb[0].dtype == torch.bfloat16


@pytest.mark.parametrize("dist", ["exp", "halfnormal"])
def test_exponential_and_half_normal_rank_distributions(dist):
    # closed forms over ranks j = 0..n-1 with scale 0.02 n, and drawn frequencies that follow them
    wl = synth.workload("tiny", batch=200_000, rank_dist=dist, rank_scale=0.02)
    s = synth.Sampler(wl)
    t, n = 1, wl.rows[1]
    p = s.row_probs(t).numpy()
    j = np.arange(n, dtype=np.float64)
    w = np.exp(-j / (0.02 * n)) if dist == "exp" else np.exp(-(j ** 2) / (2.0 * (0.02 * n) ** 2))
    want_sorted = w / w.sum()
    assert np.allclose(np.sort(p)[::-1], want_sorted, rtol=1e-12, atol=1e-300)
    idx, off = s.batch(0)
    a, b = int(off[t * wl.batch]), int(off[(t + 1) * wl.batch])
    cnt = np.bincount(idx[a:b].numpy(), minlength=n).astype(np.float64)
    m = b - a
    for e in np.argsort(-p)[:20]:
        assert abs(cnt[e] - m * p[e]) < 5 * math.sqrt(m * p[e] * (1 - p[e]))
    # almost all mass sits in the first few scale lengths: rows far down the ranking are never drawn
    cold = np.argsort(-p)[int(0.5 * n):]
    assert cnt[cold].sum() == 0
