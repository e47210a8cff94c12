"""Set-up shared by the GPU parity tests: pinned tables, a bound handle, and the oracle run beside it.

The oracle side works on its own host copies of the tables; the HIP side works on pinned copies and device
buffers.  Inputs (tables, batches, gradients) come from `synth` only.
"""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2411_01611_amd import binding, synth
from util import np_tables

RTOL, ATOL = 1e-5, 1e-6   # fp32 tolerance of the parity bar


class GpuCase:
    def __init__(self, wl: synth.Workload, budget_bytes=None, nprofile: int = 4, max_L: int = 0, state_init: float = 0.0):
        self.wl = wl
        self.dev = torch.device("cuda:0")
        self.sampler = synth.Sampler(wl)
        self.budget = wl.budget_bytes if budget_bytes is None else int(budget_bytes)
        tabs = synth.make_tables_cpu(wl)
        self.ora_tables = [x.copy() for x in np_tables(wl, tabs)]
        npdt = np.float32 if wl.dtype == "f32" else np.uint16
        self.pinned = []
        for a in self.ora_tables:
            p = binding.PinnedArray(a.shape, npdt)
            p.np[...] = a
            self.pinned.append(p)
        self.ora_state = self.pinned_state = None
        if wl.optimizer == "adagrad":
            self.ora_state = [np.full(a.shape, state_init, dtype=np.float32) for a in self.ora_tables]
            self.pinned_state = []
            for a in self.ora_state:
                p = binding.PinnedArray(a.shape, np.float32)
                p.np[...] = a
                self.pinned_state.append(p)
        self.opt = binding.OPT_ADAGRAD if wl.optimizer == "adagrad" else binding.OPT_SGD
        self.s = binding.Scars(wl.rows, wl.dim, binding.DTYPE_F32 if wl.dtype == "f32" else binding.DTYPE_BF16,
                               [p.ptr for p in self.pinned], self.opt,
                               [p.ptr for p in self.pinned_state] if self.pinned_state else None)
        # profile batches (host copies for the oracle, device copies for the library)
        self.profile = [self.sampler.batch(p, True) for p in range(nprofile)]
        self.batch = self.sampler.batch(0)
        Lmax = max([int(b[0].numel()) for b in self.profile + [self.batch]] + [max_L, 1])
        self.s.bind_buffers(self.budget, Lmax, wl.num_bags)
        self.k = None

    # ---- both sides of build_cache -------------------------------------------------------------------
    def build(self):
        """Histogram the profile batches and select the hot set, on the oracle and on the GPU."""
        wl = self.wl
        counts = np.zeros(wl.total_rows, dtype=np.uint32)
        n_p = len(self.profile)
        if n_p == 0:
            self.s.build_cache(None, None, 0, self.budget, 0)          # zero counts, select on them
        for n, (idx, off) in enumerate(self.profile):
            rc, counts = oracle.histogram(wl.rows, idx.numpy(), off.numpy(), wl.batch, counts)
            assert rc == 0
            d_idx, d_off = idx.to(self.dev), off.to(self.dev)
            if n_p == 1:
                mode = 0                                                # zero, add, select
            elif n == 0:
                self.s.build_cache(None, None, 0, self.budget, 0)      # zero (and a select on zeros)
                mode = 2
            else:
                mode = 1 if n == n_p - 1 else 2                         # add only ... add and select
            self.s.build_cache(d_idx, d_off, wl.batch, self.budget, mode)
        k = oracle.budget_rows(wl.total_rows, wl.row_bytes, self.budget)
        rc, hot, slot_of = oracle.hot_set(counts, k)
        assert rc == 0
        self.k, self.ora_counts, self.ora_hot, self.ora_slot_of = k, counts, hot, slot_of
        return counts, hot, slot_of

    def dev_batch(self, batch=None):
        idx, off = batch or self.batch
        return idx.to(self.dev), off.to(self.dev)

    def pinned_rows(self) -> np.ndarray:
        return np.concatenate([p.np for p in self.pinned])

    def pinned_state_rows(self) -> np.ndarray:
        return np.concatenate([p.np for p in self.pinned_state])

    def close(self):
        self.s.close()
        for p in self.pinned + (self.pinned_state or []):
            p.free()


def assert_close(got: np.ndarray, want: np.ndarray, what: str = ""):
    np.testing.assert_allclose(got, want, rtol=RTOL, atol=ATOL, err_msg=what)


def bf16_round_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit pattern, round to nearest even, via torch's cast (test-side helper)."""
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def assert_bf16_within(got_bits: np.ndarray, want_f64: np.ndarray, what: str = ""):
    """Each stored bf16 must be the rounding of some value within the fp32 tolerance of the oracle's
    pre-rounding value (two neighbours are both right when that value sits next to a rounding midpoint)."""
    tol = RTOL * np.abs(want_f64) + ATOL
    lo = bf16_round_bits((want_f64 - tol).astype(np.float32)).astype(np.uint32) << 16
    hi = bf16_round_bits((want_f64 + tol).astype(np.float32)).astype(np.uint32) << 16
    g = (got_bits.astype(np.uint32) << 16).view(np.float32)
    ok = (g >= lo.view(np.float32)) & (g <= hi.view(np.float32))
    assert ok.all(), f"{what}: {np.count_nonzero(~ok)} bf16 values outside the admissible rounding interval"
