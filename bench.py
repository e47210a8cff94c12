#!/usr/bin/env python3
"""Benchmark of the cached embedding-bag hot path on one MI355X.

A "step" is one pass of the whole path over one synthetic batch: remap -> embedding_bag_fwd ->
embedding_bag_bwd_update, with the workload's byte budget (hot rows in the HBM cache, cold rows in pinned host
memory).  build_cache runs once before the timed region (it is amortised over many batches) and is reported
separately.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--scale S] [--no-resident] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2411_01611_amd import binding, synth  # noqa: E402

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published
PRESORT_MIN_L = 1 << 17  # batches this large start the backward sort in remap, on the library's side stream


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


class Bench:
    def __init__(self, wl: synth.Workload, budget_bytes: int, coalesce: bool = False):
        self.wl = wl
        self.coalesce = coalesce
        self.dev = torch.device("cuda:0")
        self.budget = budget_bytes
        t0 = time.time()
        npdt = np.float32 if wl.dtype == "f32" else np.uint16
        self.tables, self.state = [], []
        for t in range(wl.num_tables):
            p = binding.PinnedArray((wl.rows[t], wl.dim), npdt)
            self._fill(p, t)
            self.tables.append(p)
            if wl.optimizer == "adagrad":
                s = binding.PinnedArray((wl.rows[t], wl.dim), np.float32)
                self._zero(s)
                self.state.append(s)
        torch.cuda.synchronize()
        log(f"tables: {wl.total_rows} rows x {wl.row_bytes} B = {wl.total_rows * wl.row_bytes / 1e9:.2f} GB pinned "
            f"(+{len(self.state) and wl.total_rows * wl.dim * 4 / 1e9:.2f} GB state) in {time.time() - t0:.1f}s")
        self.sampler = synth.Sampler(wl, self.dev)
        self.s = binding.Scars(wl.rows, wl.dim, binding.DTYPE_F32 if wl.dtype == "f32" else binding.DTYPE_BF16,
                               [p.ptr for p in self.tables],
                               binding.OPT_ADAGRAD if wl.optimizer == "adagrad" else binding.OPT_SGD,
                               [p.ptr for p in self.state] if self.state else None)

    def _fill(self, p: binding.PinnedArray, t: int):
        wl = self.wl
        chunk = max(1, (1 << 27) // wl.dim)     # 128 Mi elements per chunk
        for r0 in range(0, wl.rows[t], chunk):
            r1 = min(wl.rows[t], r0 + chunk)
            v = synth.row_values(wl, t, r0, r1, self.dev).contiguous()
            p.copy_from_device(v.view(torch.int16) if wl.dtype == "bf16" else v, r0)
            torch.cuda.synchronize()

    def _zero(self, p: binding.PinnedArray):
        rows = p.shape[0]
        chunk = max(1, (1 << 27) // p.shape[1])
        z = torch.zeros(min(rows, chunk), p.shape[1], dtype=torch.float32, device=self.dev)
        for r0 in range(0, rows, chunk):
            r1 = min(rows, r0 + chunk)
            p.copy_from_device(z[: r1 - r0], r0)
        torch.cuda.synchronize()

    def prepare(self, n_batches: int):
        wl = self.wl
        self.batches = [self.sampler.batch(e) for e in range(n_batches)]
        self.grads = [self.sampler.grads(e) for e in range(min(n_batches, 4))]
        self.max_L = max(int(b[0].numel()) for b in self.batches)
        prof = [self.sampler.batch(p, True) for p in range(min(wl.profile_batches, 4))]
        self.max_L = max(self.max_L, max(int(b[0].numel()) for b in prof)) + 4096
        self.sizes = self.s.bind_buffers(self.budget, self.max_L, wl.num_bags)
        self.rm = self.s.new_remap_out(coalesce=self.coalesce)
        self.out = torch.empty(wl.num_bags, wl.dim, dtype=torch.float32, device=self.dev)

    def build_cache(self) -> dict:
        wl = self.wl
        P = wl.profile_batches
        torch.cuda.synchronize()
        t0 = time.time()
        gen = 0.0
        Lp = 0
        self.s.build_cache(None, None, 0, self.budget, 0)
        t_hist = 0.0
        for p in range(P):
            g0 = time.time()
            idx, off = self.sampler.batch(p, True)
            if idx.numel() > self.max_L:
                continue
            torch.cuda.synchronize()
            gen += time.time() - g0
            h0 = time.time()
            self.s.build_cache(idx, off, wl.batch, self.budget, 2)
            torch.cuda.synchronize()
            t_hist += time.time() - h0
            Lp += int(idx.numel())
        s0 = time.time()
        self.s.build_cache(None, None, 0, self.budget, 1)
        torch.cuda.synchronize()
        t_sel = time.time() - s0
        # the same selection once more with a HIP event pair around every kernel: select, rank sort and fill apart
        self.s.profile_enable(True)
        self.s.build_cache(None, None, 0, self.budget, 1)
        prof = self.s.profile_read()
        self.s.profile_enable(False)
        ms = lambda *names: sum(v["total_ms"] for n, v in prof.items() if n.startswith(names))
        t_select = ms("sel_", "win_", "scan_two", "fill") * 1e-3
        t_rank = ms("sort_", "slot_scatter") * 1e-3
        t_fill = ms("cache_fill") * 1e-3
        st = self.s.sync_status()
        assert st == 0, f"device error {st} during build_cache"
        k = self.s.cache_rows()
        return {"profile_lookups": Lp, "histogram_s": t_hist, "select_and_fill_s": t_sel, "k": k,
                "histogram_Mlookups_per_s": Lp / max(t_hist, 1e-9) / 1e6,
                "fill_host_link_GBs": k * (wl.row_bytes + (wl.dim * 4 if wl.optimizer == "adagrad" else 0)) / max(t_sel, 1e-9) / 1e9,
                "select_s": t_select, "select_Mrows_per_s": wl.total_rows / max(t_select, 1e-9) / 1e6, "rank_sort_s": t_rank,
                "fill_s": t_fill, "fill_kernel_GBs": k * (wl.row_bytes + (wl.dim * 4 if wl.optimizer == "adagrad" else 0)) / max(t_fill, 1e-9) / 1e9,
                "kernels_ms": {n: round(v["total_ms"], 4) for n, v in prof.items()}, "total_s": t_hist + t_sel}

    def step(self, e: int):
        wl = self.wl
        idx, off = self.batches[e % len(self.batches)]
        g = self.grads[e % len(self.grads)]
        self.s.remap(idx, off, wl.batch, self.rm)
        self.s.embedding_bag_fwd(idx, off, wl.batch, self.rm, self.out)
        self.s.embedding_bag_bwd_update(idx, off, wl.batch, self.rm, g, wl.lr, wl.eps if wl.optimizer == "adagrad" else 0.0)
        return int(idx.numel())

    def fwd_only(self, e: int):
        idx, off = self.batches[e % len(self.batches)]
        self.s.remap(idx, off, self.wl.batch, self.rm)
        self.s.embedding_bag_fwd(idx, off, self.wl.batch, self.rm, self.out)

    def close(self):
        self.s.close()
        for p in self.tables + self.state:
            p.free()


def measure_link(dev) -> dict:
    """Pinned <-> device hipMemcpyAsync of 1 GiB: each way alone, and both ways at once on two streams (the rate each
    direction keeps while the other is busy): the host-link denominators."""
    n = 1 << 30
    host = binding.PinnedArray((n,), np.uint8)
    host2 = binding.PinnedArray((n,), np.uint8)
    d = torch.empty(n, dtype=torch.uint8, device=dev)
    d2 = torch.empty(n, dtype=torch.uint8, device=dev)
    out = {}
    for name, kind, dst, src in (("h2d_GBs", 1, d.data_ptr(), host.ptr), ("d2h_GBs", 2, host.ptr, d.data_ptr())):
        best = 0.0
        for _ in range(3):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            binding.memcpy(dst, src, n, kind)
            b.record()
            torch.cuda.synchronize()
            best = max(best, n / (a.elapsed_time(b) * 1e-3) / 1e9)
        out[name] = best
    # two streams of this measurement's own, destroyed afterwards: a process has few hardware queues, and streams left
    # behind here would push the library's side streams onto the queue of the stream the benchmark runs on
    import ctypes
    hip = ctypes.CDLL("libamdhip64.so")
    raw = [ctypes.c_void_p(), ctypes.c_void_p()]
    for r in raw:
        assert hip.hipStreamCreateWithFlags(ctypes.byref(r), 1) == 0
    s1, s2 = torch.cuda.ExternalStream(raw[0].value), torch.cuda.ExternalStream(raw[1].value)
    best_in = best_out = 0.0
    for _ in range(3):
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        with torch.cuda.stream(s1):
            ev[0].record()
            binding.memcpy(d.data_ptr(), host.ptr, n, 1)
            ev[1].record()
        with torch.cuda.stream(s2):
            ev[2].record()
            binding.memcpy(host2.ptr, d2.data_ptr(), n, 2)
            ev[3].record()
        torch.cuda.synchronize()
        best_in = max(best_in, n / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e9)
        best_out = max(best_out, n / (ev[2].elapsed_time(ev[3]) * 1e-3) / 1e9)
    del s1, s2, ev
    torch.cuda.synchronize()
    for r in raw:
        assert hip.hipStreamDestroy(r) == 0
    out["h2d_duplex_GBs"], out["d2h_duplex_GBs"] = best_in, best_out
    host.free()
    host2.free()
    return out


def calibration(dev) -> dict:
    """Plain copy kernel of known size (1 GiB read + 1 GiB write): scales the HBM byte counters and gives the
    box's own streaming rate beside the published peak."""
    n = 1 << 30
    a = torch.empty(n, dtype=torch.uint8, device=dev)
    b = torch.zeros(n, dtype=torch.uint8, device=dev)
    best = 0.0
    for _ in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        binding.calibration_copy(a, b)
        e1.record()
        torch.cuda.synchronize()
        best = max(best, 2 * n / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    sink = torch.empty(binding.CALIB_SINK_BYTES, dtype=torch.uint8, device=dev)
    best_r = 0.0
    for _ in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        binding.calibration_read(a, sink)
        e1.record()
        torch.cuda.synchronize()
        best_r = max(best_r, n / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    return {"copy_bytes_each_way": n, "copy_GBs": best, "read_GBs": best_r}


def algorithmic_bytes(wl: synth.Workload, L: float, U: float, n_miss: float) -> dict:
    """Bytes the method itself must move per launch of each kernel (per-lookup figures times the batch)."""
    R, D, G = wl.row_bytes, wl.dim, wl.num_bags
    st = 8 * D if wl.optimizer == "adagrad" else 0
    return {
        "pool_wave": L * R + G * D * 4 + 4 * L + 4 * (G + 1),
        "pool_group": L * R + G * D * 4 + 4 * L + 4 * (G + 1),
        "pool_short": L * R + G * D * 4 + 4 * L + 4 * (G + 1),
        "stage_misses": 2 * n_miss * R + 4 * n_miss,          # link read + HBM write
        "seg_rows": L * D * 4 + 8 * L + U * (2 * R + st + 12),   # with seg_long: gradient rows + row read-modify-write
        "seg_rows_long": L * D * 4 + 8 * L + U * (2 * R + st + 12),   # small batches: both in one launch
        "remap_probe": 16 * L,
        "remap_write": 8 * L + 4 * L + 4 * n_miss * 2 + 4 * (L - n_miss),
        "sort_scatter": 16 * L,
        "sort_hist": 4 * L,
        "bwd_pairs": 12 * L,
    }


def run_leg(b: Bench, K: int, W: int, link: dict, use_graph: bool = False) -> dict:
    """W warm-up steps, exactly K timed steps between two synchronizes, then the same K steps again with a HIP
    event pair around every kernel launch (recorded by the library on the launch stream)."""
    wl = b.wl
    for e in range(W):
        b.step(e)
    torch.cuda.synchronize()
    lookups = 0
    if use_graph:
        # the K steps allocate nothing and never wait on the host: capture them once, time one replay
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                for e in range(W, W + K):
                    lookups += b.step(e)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        g.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        del g
    else:
        t0 = time.perf_counter()
        for e in range(W, W + K):
            lookups += b.step(e)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    assert b.s.sync_status() == 0
    n_hit, n_miss = b.rm.n_hit_miss.cpu().tolist()
    n_staged = b.rm.n_unique_miss.cpu().tolist()[0] if b.coalesce else n_miss   # rows fetched over the link

    b.s.profile_enable(True)
    for e in range(W, W + K):
        b.step(e)
    prof = b.s.profile_read()
    b.s.profile_enable(False)
    # unique rows (all / not cached) of the last batch, for the bytes of the segment kernel
    bo = b.s.new_bwd_out()
    idx, off = b.batches[(W + K - 1) % len(b.batches)]
    b.s.embedding_bag_bwd_update(idx, off, wl.batch, b.rm, b.grads[0], wl.lr, wl.eps, bo)
    U = int(bo.n_unique.cpu()[0])
    U_cold = int((b.s.slot_of()[bo.unique_gid[:U].long()] < 0).sum().item())
    torch.cuda.synchronize()
    del bo
    # the gather kernel without the update kernel before it: inside a step it also pays for the write-back of the
    # rows the previous backward pass left dirty in the caches, so its own rate is measured on remap + forward only
    b.s.set_tuning(binding.TUNE_PRESORT, 0)     # no backward pass follows: nothing to prepare beside the forward pass
    for e in range(W):
        b.fwd_only(e)
    b.s.profile_enable(True)
    for e in range(W, W + K):
        b.fwd_only(e)
    prof_fwd = b.s.profile_read()
    # ... and with cold caches: a 1 GiB read-only sweep between remap and forward evicts L2 and Infinity Cache
    sweep = torch.empty(1 << 30, dtype=torch.uint8, device=b.dev)
    sink = torch.empty(binding.CALIB_SINK_BYTES, dtype=torch.uint8, device=b.dev)
    for e in range(W, W + K):
        idx, off = b.batches[e % len(b.batches)]
        b.s.remap(idx, off, wl.batch, b.rm)
        binding.calibration_read(sweep, sink)
        b.s.embedding_bag_fwd(idx, off, wl.batch, b.rm, b.out)
    prof_cold = b.s.profile_read()
    b.s.profile_enable(False)
    # each call alone: device-wide synchronisation around every call, side-stream option off
    alone = {"remap": 0.0, "embedding_bag_fwd": 0.0, "embedding_bag_bwd_update": 0.0}
    for e in range(W, W + K):
        idx, off = b.batches[e % len(b.batches)]
        g = b.grads[e % len(b.grads)]
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        b.s.remap(idx, off, wl.batch, b.rm)
        torch.cuda.synchronize()
        c1 = time.perf_counter()
        b.s.embedding_bag_fwd(idx, off, wl.batch, b.rm, b.out)
        torch.cuda.synchronize()
        c2 = time.perf_counter()
        b.s.embedding_bag_bwd_update(idx, off, wl.batch, b.rm, g, wl.lr, wl.eps if wl.optimizer == "adagrad" else 0.0)
        torch.cuda.synchronize()
        c3 = time.perf_counter()
        alone["remap"] += (c1 - c0) * 1e3 / K
        alone["embedding_bag_fwd"] += (c2 - c1) * 1e3 / K
        alone["embedding_bag_bwd_update"] += (c3 - c2) * 1e3 / K
    b.s.set_tuning(binding.TUNE_PRESORT, PRESORT_MIN_L if b.presort else 0)
    del sweep, sink
    # per-step spread: the same K steps once more, each between its own pair of events
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(K)]
    for i, e in enumerate(range(W, W + K)):
        evs[i][0].record()
        b.step(e)
        evs[i][1].record()
    torch.cuda.synchronize()
    per_step = sorted(a.elapsed_time(c) for a, c in evs)

    L_avg = lookups / K
    alg = algorithmic_bytes(wl, L_avg, U, n_miss)
    if "pool_short_staged" in prof:
        # one index per bag, side-stream option: bags whose row is cached are pooled by one launch while the missed
        # rows are fetched, the others by a second launch after the fetch; the bytes split with the bags
        whole = alg["pool_short"]
        alg["pool_short"] = whole * n_hit / max(1, n_hit + n_miss)
        alg["pool_short_staged"] = whole - alg["pool_short"]
    if "bwd_pairs" not in prof:
        alg["remap_write"] += alg["bwd_pairs"]   # the launch that lists hits and misses also wrote the backward pairs
    kern = {}
    for name, r in prof.items():
        avg_ms = r["total_ms"] / r["launches"]
        kern[name] = {"launches_per_step": r["launches"] / K, "avg_ms": round(avg_ms, 5),
                      "ms_per_step": round(r["total_ms"] / K, 5)}
        if name in alg:
            kern[name]["alg_GBs"] = round(alg[name] / (avg_ms * 1e-3) / 1e9, 1)
    pool = [n for n in ("pool_wave", "pool_group", "pool_short") if n in prof][0]
    pool_avg_s = prof[pool]["total_ms"] / prof[pool]["launches"] * 1e-3
    achieved = alg[pool] / pool_avg_s / 1e9
    roofline = {"kernel": pool, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": pmc_traffic(wl.name, pool),
                "alg_bytes_per_launch": int(alg[pool]), "avg_launch_ms": round(pool_avg_s * 1e3, 5)}
    alone_s = prof_fwd[pool]["total_ms"] / prof_fwd[pool]["launches"] * 1e-3
    roofline["forward_alone"] = {"avg_launch_ms": round(alone_s * 1e3, 5), "achieved": round(alg[pool] / alone_s / 1e9, 1),
                                 "frac": round(alg[pool] / alone_s / 1e9 / HBM_PEAK_GBS, 4)}
    cold_s = prof_cold[pool]["total_ms"] / prof_cold[pool]["launches"] * 1e-3
    roofline["forward_cold_caches"] = {"avg_launch_ms": round(cold_s * 1e3, 5), "achieved": round(alg[pool] / cold_s / 1e9, 1),
                                       "frac": round(alg[pool] / cold_s / 1e9 / HBM_PEAK_GBS, 4)}
    calls = {c: round(v, 5) for c, v in alone.items()}
    host_link = []
    state_b = wl.dim * 4 if wl.optimizer == "adagrad" else 0
    # forward: every missed lookup's row is read over the link.  backward: a cold row's value comes from the copy
    # the forward pass staged, so only its accumulator is read over the link; row and accumulator are written back
    for name, rd, wr in (("stage_misses", n_staged * wl.row_bytes, 0),
                         ("seg_rows", U_cold * state_b, U_cold * (wl.row_bytes + state_b)),
                         ("seg_rows_long", U_cold * state_b, U_cold * (wl.row_bytes + state_b))):
        if name in prof and rd + wr > 0:
            t_s = prof[name]["total_ms"] / prof[name]["launches"] * 1e-3
            t_min = max(rd / (link["h2d_GBs"] * 1e9), wr / (link["d2h_GBs"] * 1e9))
            host_link.append({"kernel": name, "link_read_bytes": int(rd), "link_write_bytes": int(wr),
                              "avg_launch_ms": round(t_s * 1e3, 5), "read_GBs": round(rd / t_s / 1e9, 2),
                              "write_GBs": round(wr / t_s / 1e9, 2), "frac_of_measured_link": round(t_min / t_s, 4)})
    return {"value": lookups / (t1 - t0), "ms_per_step": (t1 - t0) * 1e3 / K, "lookups_per_step": L_avg,
            "hit_rate": n_hit / max(1, n_hit + n_miss), "U": U, "U_cold": U_cold, "n_miss": n_miss, "n_staged": n_staged, "roofline": roofline,
            "host_link": host_link, "kernels": kern, "calls_alone_ms": calls,
            "ms_per_step_median": round(per_step[len(per_step) // 2], 5), "ms_per_step_min": round(per_step[0], 5),
            "_alg": alg, "_pool": pool, "_link_bytes": {"fetch": n_staged * wl.row_bytes, "acc": U_cold * state_b,
                                                        "write": U_cold * (wl.row_bytes + state_b)}}


def run_lookahead(b: Bench, K: int, W: int, leg: dict, link: dict) -> dict:
    """The same K batches in the look-ahead order: remap(e+1), update of batch e with the missed rows of batch e+1
    fetched beside it, forward pass of batch e+1.  Every batch still goes through remap, forward and update once,
    and every result is the one of the plain order (tests/test_gpu_lookahead.py)."""
    wl, s = b.wl, b.s
    n = len(b.batches)
    eps = wl.eps if wl.optimizer == "adagrad" else 0.0
    rms = [b.rm, s.new_remap_out()]
    s.set_tuning(binding.TUNE_LOOKAHEAD, 1)

    def prime(e):
        idx, off = b.batches[e % n]
        s.remap(idx, off, wl.batch, rms[e % 2])
        s.embedding_bag_fwd(idx, off, wl.batch, rms[e % 2], b.out)

    def step(e):
        idx, off = b.batches[e % n]
        nidx, noff = b.batches[(e + 1) % n]
        s.remap(nidx, noff, wl.batch, rms[(e + 1) % 2])
        s.embedding_bag_bwd_update_ahead(idx, off, wl.batch, rms[e % 2], b.grads[e % len(b.grads)], wl.lr, eps,
                                         rms[(e + 1) % 2], nidx, noff, wl.batch)
        s.embedding_bag_fwd(nidx, noff, wl.batch, rms[(e + 1) % 2], b.out)
        return int(idx.numel())

    prime(0)
    for e in range(W):
        step(e)
    torch.cuda.synchronize()
    used0 = s.get_counter(binding.COUNTER_AHEAD_USED)
    lookups = 0
    t0 = time.perf_counter()
    for e in range(W, W + K):
        lookups += step(e)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    used = s.get_counter(binding.COUNTER_AHEAD_USED) - used0
    assert s.sync_status() == 0
    s.profile_enable(True)
    for e in range(W + K, W + 2 * K):
        step(e)
    prof = s.profile_read()
    s.profile_enable(False)
    s.set_tuning(binding.TUNE_LOOKAHEAD, 0)
    s.remap(*b.batches[0], wl.batch, b.rm)      # leave no look-ahead state behind for the legs that follow
    torch.cuda.synchronize()
    kern = {k: {"launches_per_step": v["launches"] / K, "avg_ms": round(v["total_ms"] / v["launches"], 5)}
            for k, v in prof.items()}
    # the gather kernel inside this order, against the same algorithmic bytes as in the plain order
    alg, pool = leg["_alg"], leg["_pool"]
    pool_s = prof[pool]["total_ms"] / prof[pool]["launches"] * 1e-3
    roofline = {"kernel": pool, "bound": "hbm", "achieved": round(alg[pool] / pool_s / 1e9, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(alg[pool] / pool_s / 1e9 / HBM_PEAK_GBS, 4), "traffic": pmc_traffic(wl.name, pool),
                "alg_bytes_per_launch": int(alg[pool]), "avg_launch_ms": round(pool_s * 1e3, 5)}
    # the link while the update runs: the fetch for the next batch and the accumulators come in, rows and
    # accumulators go out, at the same time
    lb = leg["_link_bytes"]
    upd = "seg_rows_long" if "seg_rows_long" in prof else "seg_rows"
    t_upd = max(prof[upd]["total_ms"] / prof[upd]["launches"],
                prof["fetch_ahead"]["total_ms"] / prof["fetch_ahead"]["launches"] if "fetch_ahead" in prof else 0.0) * 1e-3
    rd, wr = lb["fetch"] + lb["acc"], lb["write"]
    host_link = [{"kernel": upd + " beside fetch_ahead", "link_read_bytes": int(rd), "link_write_bytes": int(wr),
                  "avg_launch_ms": round(t_upd * 1e3, 5), "read_GBs": round(rd / t_upd / 1e9, 2),
                  "write_GBs": round(wr / t_upd / 1e9, 2),
                  "frac_of_measured_link": round(max(rd / (link["h2d_GBs"] * 1e9), wr / (link["d2h_GBs"] * 1e9)) / t_upd, 4),
                  "frac_of_measured_duplex_link": round(max(rd / (link["h2d_duplex_GBs"] * 1e9),
                                                            wr / (link["d2h_duplex_GBs"] * 1e9)) / t_upd, 4)}]
    return {"value": lookups / (t1 - t0), "unit": "lookups/s", "ms_per_step": (t1 - t0) * 1e3 / K,
            "forward_passes_with_rows_fetched_ahead": int(used), "steps": K,
            "order": "remap(e+1) -> embedding_bag_bwd_update_ahead(e, e+1) -> embedding_bag_fwd(e+1)",
            "roofline": roofline, "host_link": host_link, "kernels": kern}


def pmc_traffic(workload: str, kernel: str):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary of this workload, if any."""
    path = os.path.join(ROOT, "profiles", f"pmc_{workload}.json")
    try:
        return json.load(open(path))[kernel]["hbm_bytes_per_launch"]
    except Exception:
        return None


def cpu_baseline(b: Bench, seconds_target: float = 12.0) -> dict:
    """The CPU oracle, as it stands, on the machine's host cores, on a bounded sample of the same workload."""
    import oracle
    wl = b.wl
    cores = min(16, os.cpu_count() or 1)
    used = oracle.set_threads(cores)
    tabs = [p.np for p in b.tables]
    st = [p.np for p in b.state] if b.state else None
    opt = 1 if wl.optimizer == "adagrad" else 0
    slot_of = b.s.slot_of().cpu().numpy()

    def run(seconds: float, max_batches: int):
        done_L, t_total, nb = 0, 0.0, 0
        while t_total < seconds and nb < max_batches:
            idx, off = b.batches[nb % len(b.batches)]
            idx, off = idx.cpu().numpy(), off.cpu().numpy()
            g = b.grads[nb % len(b.grads)].cpu().numpy()
            t0 = time.time()
            rc1 = oracle.remap(wl.rows, idx, off, wl.batch, slot_of)[0]
            rc2 = oracle.embedding_bag_fwd(wl.rows, tabs, idx, off, wl.batch)[0]
            # report mode with no output arrays: everything is computed, nothing is stored or mutated
            r = oracle.embedding_bag_bwd_update(wl.rows, tabs, st, opt, idx, off, wl.batch, g, wl.lr, wl.eps,
                                                report=True, n_unique=0, want_outputs=False)
            t_total += time.time() - t0
            assert rc1 == 0 and rc2 == 0 and r[0] == 0
            done_L += idx.shape[0]
            nb += 1
        return done_L, t_total, nb

    done_L, t_total, nb = run(seconds_target, 400)
    oracle.set_threads(1)
    one_L, one_t, one_nb = run(4.0, 50)
    oracle.set_threads(cores)
    model = "unknown"
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    return {"value": done_L / t_total, "unit": "lookups/s", "cores": used, "kind": "oracle",
            "sample": f"{nb} batch(es) of the same workload ({done_L} lookups): oracle remap + fwd + bwd_update "
                      f"(report mode, nothing mutated) in {t_total:.1f}s",
            "value_1_thread": one_L / one_t, "sample_1_thread": f"{one_nb} batch(es) in {one_t:.1f}s",
            "cpu_model": model, "host_cpus_visible": os.cpu_count()}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="multi_hot", choices=synth.WORKLOAD_NAMES)
    ap.add_argument("--scale", type=float, default=1.0)
    ap.add_argument("--row-scale", type=float, default=None,
                    help="shrink table rows and budget only (default 1.0; 0.5 for host_spill, whose 102 GB of "
                         "tables exceed what one box lets a process pin, about 64 GB)")
    ap.add_argument("--budget-bytes", type=int, default=-1, help="override the workload's cache budget")
    ap.add_argument("--also", default="dlrm_onehot,low_skew,host_spill",
                    help="comma-separated other workloads to run briefly afterwards and report under other_workloads "
                         "('none' to skip)")
    ap.add_argument("--graph", action="store_true",
                    help="capture the K timed steps into one HIP graph and time its replay instead of K eager steps")
    ap.add_argument("--coalesce", action="store_true",
                    help="remap lists each distinct missed row once (Section II-A): one link read per unique cold row")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--fused-long-max-l", type=int, default=-1,
                    help="largest batch (lookups) whose backward pass updates long runs and the other rows in one "
                         "launch (default: the library's, every batch; 0 = never)")
    ap.add_argument("--update-max-blocks", type=int, default=0,
                    help="most workgroups of the per-row update kernel (default: the library's, 8192)")
    ap.add_argument("--no-lookahead", dest="lookahead", action="store_false",
                    help="skip the extra leg in the look-ahead call order (reported under lookahead)")
    ap.add_argument("--no-presort", dest="presort", action="store_false",
                    help="sort the backward pass's (row, bag) pairs inside bwd_update instead of starting that sort in "
                         "remap on the library's side stream, beside the forward pass")
    ap.set_defaults(presort=True, lookahead=True)
    ap.add_argument("--no-resident", dest="resident", action="store_false",
                    help="skip the second leg in which every row is cached (the paper's 'hot' iteration): same "
                         "kernels, no host-link traffic; reported under cache_resident")
    ap.add_argument("--resident", dest="resident", action="store_true", help="(default) run that second leg")
    ap.set_defaults(resident=True)
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    assert torch.cuda.is_available(), "no GPU visible"
    binding.lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cal = calibration(dev)
    link = measure_link(dev)
    log("calibration", cal, "link", link)
    line = run_workload(args.workload, args, args.steps, args.warmup, cal, link, not args.no_cpu_baseline, args.resident)
    others = {}
    for name in [w for w in args.also.split(",") if w and w != "none" and w != args.workload]:
        # the other single-GPU workloads, shorter: parity-sized and link/latency-bound cases for context
        torch.cuda.empty_cache()
        r = run_workload(name, args, min(args.steps, 10), min(args.warmup, 3), cal, link, False, False)
        others[name] = {"value": r["value"], "unit": r["unit"], "ms_per_step": r["ms_per_step"], "dtype": r["dtype"],
                        "config": {k: r["config"][k] for k in ("row_scale", "rows", "dim", "batch", "lookups_per_step",
                                                                "hit_rate", "budget_bytes", "optimizer")},
                        "roofline": r["roofline"], "host_link": r["host_link"], "call_order": r["config"]["step"].split("call order: ")[1],
                        "plain_order": {k: r["plain_order"][k] for k in ("value", "ms_per_step")},
                        "lookahead": r["lookahead"] and {k: r["lookahead"][k] for k in ("value", "ms_per_step")}}
    line["other_workloads"] = others
    if args.also != "none" and args.workload != "low_skew_uniform":
        # the gather roofline reference: uniform ids over 6.4 GB of rows, every row cached (no reuse for the caches
        # to serve, so algorithmic bytes are close to HBM bytes)
        torch.cuda.empty_cache()
        r = run_workload("low_skew_uniform", args, min(args.steps, 10), min(args.warmup, 3), cal, link, False, False, True)
        line["gather_reference"] = {"workload": "low_skew_uniform, every row cached", "value": r["value"], "unit": r["unit"],
                                    "ms_per_step": r["ms_per_step"], "roofline": r["roofline"]}
    print(json.dumps(line), flush=True)


def run_workload(name: str, args, K: int, W: int, cal: dict, link: dict, with_cpu: bool, with_resident: bool,
                 all_cached: bool = False) -> dict:
    dev = torch.device("cuda:0")
    row_scale = args.row_scale if args.row_scale is not None else (0.5 if name == "host_spill" else 1.0)
    wl = synth.workload(name, scale=args.scale, row_scale=row_scale)
    budget = wl.budget_bytes if (args.budget_bytes < 0 or name != args.workload) else args.budget_bytes
    if all_cached:
        budget = wl.total_rows * wl.row_bytes

    b = Bench(wl, budget, args.coalesce)
    b.presort = bool(args.presort)
    b.s.set_tuning(binding.TUNE_PRESORT, PRESORT_MIN_L if b.presort else 0)
    if args.fused_long_max_l >= 0:
        b.s.set_tuning(binding.TUNE_FUSED_LONG_MAX_L, args.fused_long_max_l)
    if args.update_max_blocks > 0:
        b.s.set_tuning(binding.TUNE_UPDATE_MAX_BLOCKS, args.update_max_blocks)
    b.prepare(K + W)
    bc = b.build_cache()
    log(name, "build_cache", bc)

    leg = run_leg(b, K, W, link, args.graph)
    ahead = None
    if args.lookahead and not args.coalesce and budget < wl.total_rows * wl.row_bytes:
        ahead = run_lookahead(b, K, W, leg, link)
        log(name, "look-ahead order", {k: ahead[k] for k in ("value", "ms_per_step")})
    resident = None
    if with_resident and budget < wl.total_rows * wl.row_bytes and wl.total_rows * wl.row_bytes * 3 < 150e9:
        # second leg: every row cached (the paper's "hot" iteration): the same kernels, no host-link traffic
        b.s.flush_cache()
        torch.cuda.synchronize()
        b.budget = wl.total_rows * wl.row_bytes
        b.prepare(K + W)
        b.s.build_cache(None, None, 0, b.budget, 0)
        torch.cuda.synchronize()
        r = run_leg(b, K, W, link, args.graph)
        resident = {"value": r["value"], "unit": "lookups/s", "ms_per_step": r["ms_per_step"],
                    "ms_per_step_median": r["ms_per_step_median"], "ms_per_step_min": r["ms_per_step_min"],
                    "cached_rows": b.s.cache_rows(), "roofline": r["roofline"], "calls_alone_ms": r["calls_alone_ms"],
                    "kernels": r["kernels"]}
        log(name, "cache-resident leg", {k: resident[k] for k in ("value", "ms_per_step")})

    cpu = None
    b.s.flush_cache()           # host tables current again before the oracle reads them
    torch.cuda.synchronize()
    if with_cpu:
        cpu = cpu_baseline(b)
        log(name, "cpu_baseline", cpu)
    log(name, "lookups/s", f"{leg['value']:.4g}", "ms/step", f"{leg['ms_per_step']:.4f}")

    plain = {"value": leg["value"], "unit": "lookups/s", "ms_per_step": leg["ms_per_step"],
             "ms_per_step_median": leg["ms_per_step_median"], "ms_per_step_min": leg["ms_per_step_min"],
             "order": "remap(e) -> embedding_bag_fwd(e) -> embedding_bag_bwd_update(e)",
             "roofline": leg["roofline"], "host_link": leg["host_link"], "calls_alone_ms": leg["calls_alone_ms"],
             "kernels": leg["kernels"]}
    # the headline is the faster of the two call orders; both are reported in full (same batches, same results)
    best = ahead if (ahead is not None and ahead["value"] > leg["value"]) else plain
    line = {
        "metric": "pooled embedding lookups/sec (fwd+bwd) + achieved HBM GB/s, 1 GPU",
        "value": best["value"], "unit": "lookups/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": best["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if wl.dtype == "f32" else "bf16 storage, f32 sums", "data": "synthetic",
        "config": {"workload": wl.name, "scale": args.scale, "row_scale": row_scale, "tables": wl.num_tables, "rows": wl.total_rows,
                   "dim": wl.dim, "batch": wl.batch, "lookups_per_step": leg["lookups_per_step"], "zipf_s": wl.zipf_s,
                   "budget_bytes": budget, "cached_rows": bc["k"], "optimizer": wl.optimizer,
                   "hit_rate": leg["hit_rate"], "unique_rows_per_step": leg["U"],
                   "unique_cold_rows_per_step": leg["U_cold"], "missed_lookups_per_step": leg["n_miss"],
                   "rows_fetched_over_link_per_step": leg["n_staged"], "coalesce": args.coalesce,
                   "launch": ("hip graph of the K steps" if args.graph else "eager") +
                             (", backward sort prepared on the library's side stream" if args.presort else ""),
                   "step": "every batch goes through remap, embedding_bag_fwd and embedding_bag_bwd_update once; call order: " + best["order"]},
        "roofline": best["roofline"], "host_link": best["host_link"],
        "measured": {"hbm_copy_GBs": round(cal["copy_GBs"], 1), "hbm_read_GBs": round(cal["read_GBs"], 1), "h2d_GBs": round(link["h2d_GBs"], 2),
                     "d2h_GBs": round(link["d2h_GBs"], 2), "h2d_duplex_GBs": round(link["h2d_duplex_GBs"], 2),
                     "d2h_duplex_GBs": round(link["d2h_duplex_GBs"], 2)},
        "cpu_baseline": cpu, "cache_resident": resident, "plain_order": plain, "lookahead": ahead,
        "kernels": best["kernels"], "build_cache": {k: (round(v, 4) if isinstance(v, float) else v) for k, v in bc.items()},
    }
    if best is ahead:      # the gather kernel alone and with cold caches do not depend on the call order
        line["roofline"] = dict(ahead["roofline"], forward_alone=leg["roofline"]["forward_alone"],
                                forward_cold_caches=leg["roofline"]["forward_cold_caches"])
    b.close()
    del b
    return line


if __name__ == "__main__":
    main()
