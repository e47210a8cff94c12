"""Seeded synthetic workloads: table sizes, skewed index batches, rows, upstream gradients.

This module only draws inputs.  It holds none of the method's arithmetic (no histogram,
no ranking, no pooling, no update rule), so the CPU oracle's tests and the HIP path's
tests may both feed from it.  Every value is a pure function of (seed, stream, counter)
through a counter-based 64-bit mixer, evaluated with integer tensor ops so the same code
runs on the CPU (tests) and on the GPU (large benchmark tables).

The shapes follow the five benchmark workloads: categorical features with Zipf-skewed
ids over a permuted id space (the paper's skewed access premise, Introduction and
Section II-A where P(e) is defined), one lookup per feature per sample or multi-hot bags,
table-major CSR batches.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import Callable, Dict, List, Optional, Tuple

import numpy as np
import torch

_M64 = (1 << 64) - 1
_GOLD = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB

BASE_SEED = 20241101

# stream ids
S_ROWS_PER_TABLE = 1
S_PERM = 2
S_PROFILE_IDX = 3
S_EVAL_IDX = 4
S_PROFILE_LEN = 5
S_EVAL_LEN = 6
S_ROW_INIT = 7
S_GRAD = 8


def _signed(x: int) -> int:
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


def mix64_int(z: int) -> int:
    """splitmix64 output function on a Python int (reference form of `mix64`)."""
    z &= _M64
    z = ((z ^ (z >> 30)) * _C1) & _M64
    z = ((z ^ (z >> 27)) * _C2) & _M64
    return z ^ (z >> 31)


def stream_key(seed: int, stream: int, a: int = 0, b: int = 0) -> int:
    """Start state of the stream named (seed, stream, a, b)."""
    h = mix64_int(seed * _GOLD + 1)
    h = mix64_int(h ^ ((stream + 1) * _GOLD))
    h = mix64_int(h ^ ((a + 1) * _C1))
    h = mix64_int(h ^ ((b + 1) * _C2))
    return h


def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    return (z >> s) & ((1 << (64 - s)) - 1)


def mix64(z: torch.Tensor) -> torch.Tensor:
    """splitmix64 output function on int64 tensors (two's complement = mod 2^64)."""
    z = (z ^ _lsr(z, 30)) * _signed(_C1)
    z = (z ^ _lsr(z, 27)) * _signed(_C2)
    return z ^ _lsr(z, 31)


def hash_bits(key: int, counter: torch.Tensor) -> torch.Tensor:
    """64 random bits (as int64) for each counter value of stream `key`."""
    return mix64(counter.to(torch.int64) * _signed(_GOLD) + _signed(key))


def uniform01(key: int, counter: torch.Tensor) -> torch.Tensor:
    """fp64 uniform in [0, 1): top 53 bits of the hash times 2^-53."""
    return _lsr(hash_bits(key, counter), 11).to(torch.float64) * (2.0 ** -53)


# --------------------------------------------------------------------------------------
# workload descriptions
# --------------------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    name: str
    rows: Tuple[int, ...]           # N_t per table
    dim: int                        # D
    dtype: str                      # "f32" | "bf16" (storage type of rows)
    batch: int                      # B samples
    bag_lambda: Optional[float]     # None: exactly one index per (sample, table); else 1+Poisson(lambda)
    zipf_s: Optional[float]         # None: uniform ids; else bounded Zipf exponent
    budget_bytes: int               # HBM cache budget (embedding weights only)
    optimizer: str                  # "sgd" | "adagrad"
    lr: float = 0.01
    eps: float = 1e-8
    profile_batches: int = 64
    seed: int = BASE_SEED
    rank_dist: str = "zipf"         # "zipf" (exponent zipf_s; uniform ids when zipf_s is None), "exp", "halfnormal"
    rank_scale: float = 0.02        # exp: p(j) ~ exp(-j / (rank_scale * N_t)); halfnormal: p(j) ~ exp(-j^2 / (2 (rank_scale * N_t)^2))

    @property
    def num_tables(self) -> int:
        return len(self.rows)

    @property
    def total_rows(self) -> int:
        return int(sum(self.rows))

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def row_bytes(self) -> int:
        return self.dim * self.elem_bytes

    @property
    def num_bags(self) -> int:
        return self.num_tables * self.batch

    @property
    def row_base(self) -> np.ndarray:
        rb = np.zeros(self.num_tables + 1, dtype=np.int64)
        rb[1:] = np.cumsum(np.asarray(self.rows, dtype=np.int64))
        return rb

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16


def _log_uniform_rows(seed: int, T: int, lo: float, hi: float) -> List[int]:
    u = uniform01(stream_key(seed, S_ROWS_PER_TABLE), torch.arange(T)).tolist()
    a, b = math.log10(lo), math.log10(hi)
    out = []
    for x in u:
        n = int(math.floor(10.0 ** (a + (b - a) * x)))
        out.append(int(min(max(n, int(lo)), int(hi))))
    return out


def _scale_to_total(rows: List[int], total: int, lo: int, hi: int) -> List[int]:
    """Scale log-uniform draws to an exact total while keeping every table within [lo, hi]."""
    out = [float(r) for r in rows]
    fixed = [False] * len(out)
    for _ in range(len(out) + 1):
        free = [i for i in range(len(out)) if not fixed[i]]
        s = (total - sum(out[i] for i in range(len(out)) if fixed[i])) / sum(out[i] for i in free)
        clipped = False
        for i in free:
            v = out[i] * s
            if v > hi or v < lo:
                out[i] = float(min(max(v, lo), hi))
                fixed[i] = True
                clipped = True
        if not clipped:
            for i in free:
                out[i] *= s
            break
    res = [int(min(max(int(v), lo), hi)) for v in out]
    free = [i for i in range(len(res)) if not fixed[i]]
    j = max(free, key=lambda i: res[i])
    res[j] += total - sum(res)
    assert sum(res) == total and lo <= res[j] <= hi
    return res


def workload(name: str, scale: float = 1.0, seed: int = BASE_SEED, row_scale: float = 1.0, **over) -> Workload:
    """The five benchmark workloads; `scale` < 1 shrinks rows, batch and budget together, `row_scale` < 1
    shrinks rows and budget only (same batch shape, same budget-to-bytes ratio)."""
    if name == "tiny":
        rows = [10_000] * 4
        wl = Workload(name, tuple(rows), 16, "f32", 256, None, 1.05,
                      (sum(rows) // 10) * 64, "sgd", seed=seed)
    elif name == "dlrm_onehot":
        rows = _log_uniform_rows(seed, 26, 10, 10_000_000)
        wl = Workload(name, tuple(rows), 64, "f32", 2048, None, 1.1,
                      int(0.05 * sum(rows) * 256), "sgd", seed=seed)
    elif name == "multi_hot":
        rows = [5_000_000] * 8
        wl = Workload(name, tuple(rows), 128, "f32", 4096, 19.0, 0.9,
                      2_000_000_000, "adagrad", seed=seed)
    elif name == "host_spill":
        rows = _scale_to_total(_log_uniform_rows(seed, 26, 1_000, 40_000_000),
                               200_000_000, 1_000, 40_000_000)
        wl = Workload(name, tuple(rows), 128, "f32", 65_536, None, 1.2,
                      16_000_000_000, "sgd", profile_batches=16, seed=seed)
    elif name in ("multi_hot_exp", "multi_hot_halfnormal"):
        # the multi-hot shape with the paper's two other rank distributions (end of Section II-B)
        rows = [5_000_000] * 8
        wl = Workload(name, tuple(rows), 128, "f32", 4096, 19.0, None, 2_000_000_000, "adagrad", seed=seed,
                      rank_dist="exp" if name.endswith("exp") else "halfnormal", rank_scale=0.02)
    elif name in ("low_skew", "low_skew_uniform"):
        rows = _scale_to_total(_log_uniform_rows(seed, 26, 1_000, 10_000_000),
                               50_000_000, 1_000, 10_000_000)
        wl = Workload(name, tuple(rows), 64, "bf16", 16_384, 9.0,
                      0.5 if name == "low_skew" else None,
                      (sum(rows) // 10) * 128, "sgd", seed=seed)
    else:
        raise ValueError(f"unknown workload {name!r}")
    if scale != 1.0:
        rows = tuple(max(4, int(r * scale)) for r in wl.rows)
        frac = wl.budget_bytes / float(wl.total_rows * wl.row_bytes)
        wl = replace(wl, rows=rows, batch=max(8, int(wl.batch * scale)),
                     budget_bytes=int(frac * sum(rows)) * wl.row_bytes)
    if row_scale != 1.0:
        rows = tuple(max(4, int(r * row_scale)) for r in wl.rows)
        frac = wl.budget_bytes / float(wl.total_rows * wl.row_bytes)
        wl = replace(wl, rows=rows, budget_bytes=int(frac * sum(rows)) * wl.row_bytes)
    if over:
        wl = replace(wl, **over)
    return wl


WORKLOAD_NAMES = ("tiny", "dlrm_onehot", "multi_hot", "host_spill", "low_skew", "low_skew_uniform",
                  "multi_hot_exp", "multi_hot_halfnormal")


# --------------------------------------------------------------------------------------
# distributions
# --------------------------------------------------------------------------------------
def zipf_probs(n: int, s: float, device="cpu") -> torch.Tensor:
    """p(j) = j^-s / H_{n,s} for ranks j = 1..n, fp64."""
    w = torch.arange(1, n + 1, dtype=torch.float64, device=device).pow_(-s)
    return w / w.sum()


def rank_weights(n: int, dist: str, param: float, device="cpu") -> torch.Tensor:
    """Unnormalised weight of rank j = 1..n.  Zipf, exponential and half-normal are the three rank
    distributions the paper analyses at the end of Section II-B (it calls Criteo closest to half-normal)."""
    j = torch.arange(1, n + 1, dtype=torch.float64, device=device)
    if dist == "zipf":
        return j.pow_(-param)
    if dist == "exp":
        return torch.exp(-(j - 1) / (param * n))
    if dist == "halfnormal":
        return torch.exp(-((j - 1) ** 2) / (2.0 * (param * n) ** 2))
    raise ValueError(f"unknown rank distribution {dist!r}")


def _zipf_cdf(n: int, s: float, device) -> torch.Tensor:
    c = torch.cumsum(rank_weights(n, "zipf", s, device), 0)
    return c / c[-1]


def _poisson_cdf(lam: float) -> torch.Tensor:
    kmax = int(lam + 12.0 * math.sqrt(lam) + 20)
    p = [math.exp(-lam)]
    for k in range(1, kmax + 1):
        p.append(p[-1] * lam / k)
    c = np.cumsum(np.asarray(p, dtype=np.float64))
    c[-1] = 1.0
    return torch.from_numpy(c)


class Sampler:
    """Draws batches for one workload; caches each table's permutation and CDF on `device`."""

    def __init__(self, wl: Workload, device="cpu"):
        self.wl = wl
        self.device = torch.device(device)
        self._perm: Dict[int, torch.Tensor] = {}
        self._cdf: Dict[Tuple[int, float], torch.Tensor] = {}
        self._pois = _poisson_cdf(wl.bag_lambda).to(self.device) if wl.bag_lambda else None

    def permutation(self, t: int) -> torch.Tensor:
        """Seeded permutation rank -> row id of table t (stable argsort of hashed keys)."""
        if t not in self._perm:
            n = self.wl.rows[t]
            k = hash_bits(stream_key(self.wl.seed, S_PERM, t),
                          torch.arange(n, device=self.device))
            self._perm[t] = torch.argsort(k, stable=True).to(torch.int32)
        return self._perm[t]

    def _dist(self):
        wl = self.wl
        return ("zipf", wl.zipf_s) if wl.rank_dist == "zipf" else (wl.rank_dist, wl.rank_scale)

    def cdf(self, t: int) -> torch.Tensor:
        key = (self.wl.rows[t],) + self._dist()
        if key not in self._cdf:
            c = torch.cumsum(rank_weights(key[0], key[1], key[2], self.device), 0)
            self._cdf[key] = c / c[-1]
        return self._cdf[key]

    def row_probs(self, t: int) -> torch.Tensor:
        """P(e) for every row id of table t (Section II-A's P(e)), fp64, on CPU."""
        n = self.wl.rows[t]
        if self._uniform():
            return torch.full((n,), 1.0 / n, dtype=torch.float64)
        d, prm = self._dist()
        w = rank_weights(n, d, prm)
        p = torch.empty(n, dtype=torch.float64)
        p[self.permutation(t).cpu().long()] = w / w.sum()
        return p

    def _uniform(self) -> bool:
        return self.wl.rank_dist == "zipf" and self.wl.zipf_s is None

    def lengths(self, batch_id: int, t: int, profile: bool) -> torch.Tensor:
        B = self.wl.batch
        if self._pois is None:
            return torch.ones(B, dtype=torch.int64, device=self.device)
        key = stream_key(self.wl.seed, S_PROFILE_LEN if profile else S_EVAL_LEN, batch_id, t)
        u = uniform01(key, torch.arange(B, device=self.device))
        return 1 + torch.searchsorted(self._pois, u, right=True).clamp_(max=self._pois.numel() - 1)

    def batch(self, batch_id: int, profile: bool = False) -> Tuple[torch.Tensor, torch.Tensor]:
        """(indices int32 [L], offsets int32 [T*B+1]); bag g = t*B + b, table-local row ids."""
        wl = self.wl
        idx_parts, len_parts = [], []
        for t in range(wl.num_tables):
            ln = self.lengths(batch_id, t, profile)
            m = int(ln.sum().item())
            key = stream_key(wl.seed, S_PROFILE_IDX if profile else S_EVAL_IDX, batch_id, t)
            u = uniform01(key, torch.arange(m, device=self.device))
            n = wl.rows[t]
            if self._uniform():
                idx = (u * n).to(torch.int64).clamp_(max=n - 1).to(torch.int32)
            else:
                rank = torch.searchsorted(self.cdf(t), u, right=False).clamp_(max=n - 1)
                idx = self.permutation(t)[rank]
            idx_parts.append(idx)
            len_parts.append(ln)
        lens = torch.cat(len_parts)
        offsets = torch.zeros(lens.numel() + 1, dtype=torch.int64, device=self.device)
        torch.cumsum(lens, 0, out=offsets[1:])
        assert int(offsets[-1].item()) < 2 ** 31
        return torch.cat(idx_parts).contiguous(), offsets.to(torch.int32)

    def grads(self, batch_id: int) -> torch.Tensor:
        """Upstream gradient N(0,1), fp32 [T*B, D] (Box-Muller on two hashed uniforms)."""
        wl = self.wl
        n = wl.num_bags * wl.dim
        c = torch.arange(n, device=self.device)
        key = stream_key(wl.seed, S_GRAD, batch_id)
        u1 = 1.0 - uniform01(key, 2 * c)          # (0, 1]
        u2 = uniform01(key, 2 * c + 1)
        z = torch.sqrt(-2.0 * torch.log(u1)) * torch.cos(2.0 * math.pi * u2)
        return z.to(torch.float32).reshape(wl.num_bags, wl.dim)


def row_values(wl: Workload, t: int, r0: int, r1: int, device="cpu") -> torch.Tensor:
    """Rows [r0, r1) of table t: U(-0.01, 0.01) as a function of (seed, global row, column)."""
    base = int(wl.row_base[t])
    g = torch.arange(base + r0, base + r1, device=device, dtype=torch.int64)
    c = g[:, None] * wl.dim + torch.arange(wl.dim, device=device, dtype=torch.int64)[None, :]
    u = uniform01(stream_key(wl.seed, S_ROW_INIT), c)
    return ((2.0 * u - 1.0) * 0.01).to(torch.float32).to(wl.torch_dtype)


def fill_table(wl: Workload, t: int, dst: torch.Tensor, device="cpu", chunk_rows: int = 1 << 20,
               copy: Optional[Callable[[torch.Tensor, torch.Tensor], None]] = None) -> None:
    """Write table t's rows into the CPU tensor `dst` [N_t, D], generating on `device`."""
    n = wl.rows[t]
    for r0 in range(0, n, chunk_rows):
        r1 = min(n, r0 + chunk_rows)
        v = row_values(wl, t, r0, r1, device)
        if copy is not None:
            copy(dst[r0:r1], v)
        else:
            dst[r0:r1].copy_(v)


def make_tables_cpu(wl: Workload) -> List[torch.Tensor]:
    """All tables as ordinary CPU tensors (small workloads, CPU tests)."""
    out = []
    for t in range(wl.num_tables):
        w = torch.empty(wl.rows[t], wl.dim, dtype=wl.torch_dtype)
        fill_table(wl, t, w)
        out.append(w)
    return out
