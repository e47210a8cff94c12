#!/usr/bin/env python3
"""Benchmark of the cached embedding-bag hot path on one MI355X.

A "step" is one pass of the whole path over one synthetic batch: remap -> embedding_bag_fwd ->
embedding_bag_bwd_update, with the workload's byte budget (hot rows in the HBM cache, cold rows in pinned host
memory).  build_cache runs once before the timed region (it is amortised over many batches) and is reported
separately.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--scale S] [--no-resident] [--no-cpu-baseline]

What the line's `roofline` object is: the kernel that takes the largest share of the reported step, priced against
the resource that bounds it -- the host link (its measured one-way copy rate) for the kernels that move cold rows,
HBM (8 TB/s, published) for the others -- with `frac` = the bytes the method cannot avoid moving / launch time / that
rate, never above 1.  The pooled-sum (gather) kernel, the HBM-bound core of the forward pass, is reported beside it
under `gather` with three figures: compulsory bytes, effective bytes (every lookup's row counted, so repeats served
by the caches push it past the peak) and counter bytes.
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
# With every row cached the threshold gates one thing only, the look-ahead order's preparation of the next batch's sort
# beside this batch's update.  That pays from about 64k lookups (one index per bag, 26 tables: 0.107 -> 0.085 - 0.093 ms
# per step at 106k lookups; 0.077 - 0.089 against 0.082 - 0.084 at 53k, no clear gain; at 4k it costs 0.015 ms, the fork
# and join of the side stream).
PREPARE_MIN_L_CACHED = 1 << 16
POOL_KERNELS = ("pool_wave", "pool_group", "pool_short")
UPDATE_KERNELS = ("seg_rows_long+fetch_ahead", "seg_rows_long", "seg_rows", "small_update")


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def pin_tables(wl: synth.Workload, with_state: bool):
    """Pinned host arrays for every table (and accumulator) of the workload, or (None, what failed)."""
    npdt = np.float32 if wl.dtype == "f32" else np.uint16
    tables, state, done = [], [], 0
    try:
        for t in range(wl.num_tables):
            tables.append(binding.PinnedArray((wl.rows[t], wl.dim), npdt))
            done += tables[-1].nbytes
            if with_state:
                state.append(binding.PinnedArray((wl.rows[t], wl.dim), np.float32))
                done += state[-1].nbytes
    except binding.ScarsError as e:
        for p in tables + state:
            p.free()
        need = wl.total_rows * (wl.row_bytes + (wl.dim * 4 if with_state else 0))
        return None, {"pinned_bytes_wanted": int(need), "pinned_bytes_before_failure": int(done),
                      "failing_table": len(tables), "error": f"hipHostMalloc: {e}"}
    return (tables, state), None


class Bench:
    def __init__(self, wl: synth.Workload, budget_bytes: int, pinned, coalesce: bool = False):
        self.wl = wl
        self.coalesce = coalesce
        self.dev = torch.device("cuda:0")
        self.budget = budget_bytes
        t0 = time.time()
        self.tables, self.state = pinned
        for t in range(wl.num_tables):
            self._fill(self.tables[t], t)
            if self.state:
                self._zero(self.state[t])
        torch.cuda.synchronize()
        log(f"tables: {wl.total_rows} rows x {wl.row_bytes} B = {wl.total_rows * wl.row_bytes / 1e9:.2f} GB pinned "
            f"(+{len(self.state) and wl.total_rows * wl.dim * 4 / 1e9:.2f} GB state) filled in {time.time() - t0:.1f}s")
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

    def build_cache(self, link: dict) -> dict:
        """The three parts of build_cache apart, each against the bytes it has to move."""
        wl = self.wl
        P = wl.profile_batches
        R, N = wl.row_bytes, wl.total_rows
        torch.cuda.synchronize()
        Lp = 0
        self.s.build_cache(None, None, 0, self.budget, 0)
        t_hist = 0.0
        self.s.profile_enable(True)
        for p in range(P):
            idx, off = self.sampler.batch(p, True)
            if idx.numel() > self.max_L:
                continue
            torch.cuda.synchronize()
            h0 = time.time()
            self.s.build_cache(idx, off, wl.batch, self.budget, 2)
            torch.cuda.synchronize()
            t_hist += time.time() - h0
            Lp += int(idx.numel())
        hist_prof = self.s.profile_read()
        self.s.profile_enable(False)
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
        t_select = ms("sel_", "win_", "scan_two") * 1e-3
        t_rank = ms("sort_", "slot_scatter") * 1e-3
        t_fill = ms("cache_fill") * 1e-3
        st = self.s.sync_status()
        assert st == 0, f"device error {st} during build_cache"
        k = self.s.cache_rows()
        state_b = wl.dim * 4 if wl.optimizer == "adagrad" else 0
        hk = hist_prof.get("histogram", {"launches": 1, "total_ms": 0.0})
        hist_launch_s = hk["total_ms"] / max(1, hk["launches"]) * 1e-3
        Lp_launch = Lp / max(1, hk["launches"])
        # bytes each part has to move: 12 per profiled lookup (index + counter read-modify-write); one read of the
        # counts per select pass (three) and per winner pass (two) plus the slot map written once; k rows over the link
        sel_bytes = 5 * 4 * N + 4 * N + 8 * k
        fill_bytes = k * (R + state_b)
        fill_rate = fill_bytes / max(t_fill, 1e-9) / 1e9
        parts = {
            "a1_histogram": {"kernel": "histogram", "bound": "hbm", "lookups_per_launch": Lp_launch,
                             "avg_launch_ms": round(hist_launch_s * 1e3, 5), "alg_bytes_per_launch": int(12 * Lp_launch),
                             "achieved": round(12 * Lp_launch / max(hist_launch_s, 1e-12) / 1e9, 1), "peak": HBM_PEAK_GBS,
                             "unit": "GB/s", "frac": round(12 * Lp_launch / max(hist_launch_s, 1e-12) / 1e9 / HBM_PEAK_GBS, 4),
                             "Mlookups_per_s": round(Lp_launch / max(hist_launch_s, 1e-12) / 1e6, 1)},
            "a2_select": {"kernels": "sel_hist x3, sel_pick x3, win_count, scan_two, win_write", "bound": "hbm",
                          "ms": round(t_select * 1e3, 4), "alg_bytes": int(sel_bytes),
                          "achieved": round(sel_bytes / max(t_select, 1e-12) / 1e9, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                          "frac": round(sel_bytes / max(t_select, 1e-12) / 1e9 / HBM_PEAK_GBS, 4),
                          "Mrows_per_s": round(N / max(t_select, 1e-12) / 1e6, 1),
                          "rank_sort_of_the_k_winners_ms": round(t_rank * 1e3, 4)},
            "a3_fill": {"kernel": "cache_fill", "bound": "host_link", "ms": round(t_fill * 1e3, 3),
                        "link_read_bytes": int(fill_bytes), "achieved": round(fill_rate, 2), "peak": round(link["h2d_GBs"], 2),
                        "peak_source": "hipMemcpyAsync of 1 GiB pinned -> device, this run", "unit": "GB/s",
                        "frac": round(min(1.0, fill_rate / link["h2d_GBs"]), 4)},
        }
        return {"profile_lookups": Lp, "histogram_s": t_hist, "select_and_fill_s": t_sel, "k": k,
                "roofline": parts, "kernels_ms": {n: round(v["total_ms"], 4) for n, v in prof.items()},
                "total_s": t_hist + t_sel}

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


def _timed(fn, reps=3):
    best = float("inf")
    for _ in range(reps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        torch.cuda.synchronize()
        best = min(best, a.elapsed_time(b) * 1e-3)
    return best


def measure_link(dev) -> dict:
    """The host-link denominators, all measured in this run: hipMemcpyAsync of 1 GiB each way, alone and both ways at
    once; and the library's calibration kernel moving scattered pieces of 64 .. 512 bytes the way the fetch of missed
    rows (reads) and the update of cold rows (writes) do, alone and both at once."""
    n = 1 << 30
    host = binding.PinnedArray((n,), np.uint8)
    host2 = binding.PinnedArray((n,), np.uint8)
    d = torch.empty(n, dtype=torch.uint8, device=dev)
    d2 = torch.empty(n, dtype=torch.uint8, device=dev)
    out = {}
    out["h2d_GBs"] = n / _timed(lambda: binding.memcpy(d.data_ptr(), host.ptr, n, 1)) / 1e9
    out["d2h_GBs"] = n / _timed(lambda: binding.memcpy(host.ptr, d.data_ptr(), n, 2)) / 1e9
    # scattered pieces over the whole 1 GiB of host memory, 256 MiB moved per launch
    moved = 1 << 28
    rd, wr = {}, {}
    for g in (64, 128, 256, 512):
        rd[str(g)] = round(moved / _timed(lambda: binding.calibration_link(host, d, moved // g, g, True, False, 128)) / 1e9, 2)
        wr[str(g)] = round(moved / _timed(lambda: binding.calibration_link(host2, d2, moved // g, g, True, True, 512)) / 1e9, 2)
    out["link_random_read_GBs"] = rd
    out["link_random_write_GBs"] = wr
    out["link_sequential_read_512B_GBs"] = round(
        moved / _timed(lambda: binding.calibration_link(host, d, moved // 512, 512, False, False, 128)) / 1e9, 2)
    # two streams of this measurement's own, destroyed afterwards: a process has few hardware queues, and streams left
    # behind here could push the library's side streams onto the queue of the stream the benchmark runs on
    import ctypes
    hip = ctypes.CDLL("libamdhip64.so")
    raw = [ctypes.c_void_p(), ctypes.c_void_p()]
    for r in raw:
        assert hip.hipStreamCreateWithFlags(ctypes.byref(r), 1) == 0
    s1, s2 = torch.cuda.ExternalStream(raw[0].value), torch.cuda.ExternalStream(raw[1].value)

    def both(fn_in, fn_out, nbytes):
        best_in = best_out = 0.0
        for _ in range(3):
            torch.cuda.synchronize()
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
            with torch.cuda.stream(s1):
                ev[0].record()
                fn_in()
                ev[1].record()
            with torch.cuda.stream(s2):
                ev[2].record()
                fn_out()
                ev[3].record()
            torch.cuda.synchronize()
            best_in = max(best_in, nbytes / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e9)
            best_out = max(best_out, nbytes / (ev[2].elapsed_time(ev[3]) * 1e-3) / 1e9)
            del ev
        return best_in, best_out

    out["h2d_duplex_GBs"], out["d2h_duplex_GBs"] = both(lambda: binding.memcpy(d.data_ptr(), host.ptr, n, 1),
                                                          lambda: binding.memcpy(host2.ptr, d2.data_ptr(), n, 2), n)
    kin, kout = both(lambda: binding.calibration_link(host, d, moved // 512, 512, True, False, 128),
                     lambda: binding.calibration_link(host2, d2, moved // 512, 512, True, True, 512), moved)
    out["link_kernel_duplex_512B_GBs"] = {"read": round(kin, 2), "write": round(kout, 2)}
    del s1, s2
    torch.cuda.synchronize()
    for r in raw:
        assert hip.hipStreamDestroy(r) == 0
    host.free()
    host2.free()
    return out


def calibration(dev) -> dict:
    """Plain copy kernel of known size (1 GiB read + 1 GiB write): scales the HBM byte counters and gives the
    box's own streaming rate beside the published peak."""
    n = 1 << 30
    a = torch.empty(n, dtype=torch.uint8, device=dev)
    b = torch.zeros(n, dtype=torch.uint8, device=dev)
    t_copy = _timed(lambda: binding.calibration_copy(a, b))
    sink = torch.empty(binding.CALIB_SINK_BYTES, dtype=torch.uint8, device=dev)
    t_read = _timed(lambda: binding.calibration_read(a, sink))
    return {"copy_bytes_each_way": n, "copy_GBs": 2 * n / t_copy / 1e9, "read_GBs": n / t_read / 1e9}


def bytes_model(wl: synth.Workload, L: float, U: float, U_cold: float, n_miss: float, n_staged: float) -> dict:
    """Bytes per launch of each kernel: `alg` = what the kernel's own definition moves (every lookup's row counted),
    `min` = what no implementation could avoid (a row that several lookups of the batch share is counted once)."""
    R, D, G = wl.row_bytes, wl.dim, wl.num_bags
    st = 8 * D if wl.optimizer == "adagrad" else 0
    pool_alg = L * R + G * D * 4 + 4 * L + 4 * (G + 1)
    pool_min = (U - U_cold + n_staged) * R + G * D * 4 + 4 * L + 4 * (G + 1)
    upd_alg = L * D * 4 + 8 * L + U * (2 * R + st + 12)
    upd_min = min(L, G) * D * 4 + 8 * L + U * (2 * R + st + 12)
    m = {n: {"alg": pool_alg, "min": pool_min} for n in POOL_KERNELS}
    m.update({n: {"alg": upd_alg, "min": upd_min} for n in UPDATE_KERNELS})
    # the update by position reads a length and a source per position instead of the 12 bytes per run of a run list
    m["small_update"] = {"alg": upd_alg + 8 * L - 12 * U, "min": upd_min + 8 * L - 12 * U}
    m.update({
        "stage_misses": {"alg": 2 * n_staged * R + 4 * n_staged, "min": 2 * n_staged * R + 4 * n_staged},   # link read + HBM write
        "remap_probe": {"alg": 16 * L, "min": 16 * L},
        "remap_write": {"alg": 8 * L + 4 * L + 4 * n_miss * 2 + 4 * (L - n_miss), "min": 8 * L + 4 * L + 4 * n_miss * 2 + 4 * (L - n_miss)},
        "sort_scatter": {"alg": 16 * L, "min": 16 * L},
        "sort_hist": {"alg": 4 * L, "min": 4 * L},
        "bwd_pairs": {"alg": 12 * L, "min": 12 * L},
        "seg_count": {"alg": 4 * L, "min": 4 * L},
        "seg_write": {"alg": 12 * L + 20 * U, "min": 12 * L + 20 * U},
    })
    return m


def sources_sha1() -> str:
    """One hash over the library's kernel sources: the committed counter summaries record the hash they were taken
    with, so that a bench line can say when its `traffic` figures belong to other kernels than the ones it timed."""
    import hashlib
    h = hashlib.sha1()
    d = os.path.join(ROOT, "paper_2411_01611_amd", "csrc")
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(d, name), "rb").read())
    return h.hexdigest()


def pmc_sources_match(wl: synth.Workload, every_row_cached: bool = False):
    """True / False when the counter summary of this workload records the kernel sources it was taken with; else None."""
    name = f"pmc_{wl.name}_every_row_cached.json" if every_row_cached else f"pmc_{wl.name}.json"
    try:
        rec = json.load(open(os.path.join(ROOT, "profiles", name)))
    except Exception:
        try:
            rec = json.load(open(os.path.join(ROOT, "profiles", f"pmc_{wl.name}.json")))
        except Exception:
            return None
    return (rec["_sources_sha1"] == sources_sha1()) if "_sources_sha1" in rec else None


def pmc_traffic(wl: synth.Workload, kernel: str, every_row_cached: bool = False):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary of this workload (a separate run of
    the same command: the counters cannot be read from inside this process), or None.  The counters belong to the
    full-size workload with its own budget, or with every row cached: anything else gets None."""
    if wl.total_rows != synth.workload(wl.name).total_rows:
        return None
    names = [f"pmc_{wl.name}_every_row_cached.json", f"pmc_{wl.name}.json"] if every_row_cached else [f"pmc_{wl.name}.json"]
    if wl.name == "low_skew_uniform" and not every_row_cached:
        return None          # only its every-row-cached leg was profiled (profiles/pmc_low_skew_uniform.json)
    for n in names:
        try:
            return json.load(open(os.path.join(ROOT, "profiles", n)))[kernel]["hbm_bytes_per_launch"]
        except Exception:
            continue
    return None


def avg_s(prof: dict, name: str) -> float:
    return prof[name]["total_ms"] / prof[name]["launches"] * 1e-3


def hbm_roofline(name: str, t_s: float, model: dict, traffic, ms_per_step: float, launches_per_step: float,
                 sources_match=None) -> dict:
    b = model[name]
    r = {"kernel": name, "bound": "hbm", "achieved": round(b["min"] / t_s / 1e9, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
         "frac": round(min(1.0, b["min"] / t_s / 1e9 / HBM_PEAK_GBS), 4),
         "bytes_counted": "compulsory: a row shared by several lookups of the batch counted once",
         "compulsory_bytes_per_launch": int(b["min"]), "alg_bytes_per_launch": int(b["alg"]),
         "effective_GBs": round(b["alg"] / t_s / 1e9, 1), "effective_vs_peak": round(b["alg"] / t_s / 1e9 / HBM_PEAK_GBS, 4),
         "traffic": traffic, "avg_launch_ms": round(t_s * 1e3, 5),
         "share_of_step": round(t_s * 1e3 * launches_per_step / ms_per_step, 4)}
    if traffic:
        r["traffic_taken_with_these_kernel_sources"] = sources_match
        r["counter_GBs"] = round(traffic / t_s / 1e9, 1)
        r["frac_counter"] = round(traffic / t_s / 1e9 / HBM_PEAK_GBS, 4)
        r["traffic_source"] = "profiles/pmc_<workload>[_every_row_cached].json: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of a separate run of this workload (command in the file), scaled by the 1 GiB copy kernel; not measured in this process"
    return r


def link_roofline(name: str, t_s: float, rd: float, wr: float, link: dict, traffic, ms_per_step: float,
                  granule: int) -> dict:
    """A kernel bound by the host link: both directions against the measured one-way copy rates; beside them the
    rates the link gives a kernel moving scattered pieces of this row size, measured in the same run."""
    t_min = max(rd / (link["h2d_GBs"] * 1e9), wr / (link["d2h_GBs"] * 1e9))
    lead_rd = rd / link["h2d_GBs"] >= wr / link["d2h_GBs"]
    g = str(min(512, max(64, granule)))
    r = {"kernel": name, "bound": "host_link", "achieved": round((rd if lead_rd else wr) / t_s / 1e9, 2),
         "peak": round(link["h2d_GBs"] if lead_rd else link["d2h_GBs"], 2),
         "peak_source": "hipMemcpyAsync of 1 GiB, one way, measured in this run", "unit": "GB/s",
         "frac": round(min(1.0, t_min / t_s), 4), "direction_priced": "host to device" if lead_rd else "device to host",
         "link_read_bytes": int(rd), "link_write_bytes": int(wr), "read_GBs": round(rd / t_s / 1e9, 2),
         "write_GBs": round(wr / t_s / 1e9, 2), "avg_launch_ms": round(t_s * 1e3, 5),
         "share_of_step": round(t_s * 1e3 / ms_per_step, 4), "traffic": traffic,
         "row_bytes": granule,
         "measured_ceiling_for_scattered_rows_of_this_size_GBs": {"read": link["link_random_read_GBs"][g],
                                                                  "write": link["link_random_write_GBs"][g]},
         "frac_of_that_ceiling": round(min(1.0, max(rd / (link["link_random_read_GBs"][g] * 1e9),
                                                    wr / (link["link_random_write_GBs"][g] * 1e9)) / t_s), 4)}
    if rd > 0 and wr > 0:
        r["frac_of_duplex_copy"] = round(min(1.0, max(rd / (link["h2d_duplex_GBs"] * 1e9), wr / (link["d2h_duplex_GBs"] * 1e9)) / t_s), 4)
        r["request_bound"] = False
    if granule < 256:
        r["request_bound"] = True      # below 256 bytes per piece the link gives requests per second, not bytes
    return r


def rooflines(wl, prof, K, ms_per_step, model, link, link_bytes, which_pool=None, cached=False):
    """(dominant-kernel roofline, gather roofline, host_link list) of one leg from its per-kernel times."""
    pmc = lambda kernel: pmc_traffic(wl, kernel, cached)
    match = pmc_sources_match(wl, cached)
    per_step = {n: r["total_ms"] / K for n, r in prof.items()}
    dominant = max(per_step, key=per_step.get)
    pool = which_pool or [n for n in POOL_KERNELS if n in prof][0]
    gather = hbm_roofline(pool, avg_s(prof, pool), model, pmc(pool), ms_per_step, prof[pool]["launches"] / K, match)
    host_link = []
    beside = None
    for name in ("stage_misses",) + UPDATE_KERNELS:
        if name not in prof:
            continue
        rd, wr = link_bytes(name)
        if rd + wr > 0:
            t, label = avg_s(prof, name), name
            if name != "stage_misses" and "fetch_ahead" in prof:
                # the fetch for the next batch is a launch of its own on the library's stream, beside this update:
                # the pair is priced as one, over the longer of the two
                t, label = max(t, avg_s(prof, "fetch_ahead")), name + " beside fetch_ahead"
                beside = label
            host_link.append(link_roofline(label, t, rd, wr, link, pmc(name), ms_per_step, wl.row_bytes))
            if host_link[-1]["traffic"]:
                host_link[-1]["traffic_taken_with_these_kernel_sources"] = match
    by_name = {r["kernel"]: r for r in host_link}
    if beside and (dominant == "fetch_ahead" or dominant + " beside fetch_ahead" == beside):
        dominant = beside
    if dominant in by_name:
        top = by_name[dominant]
    elif dominant in model:
        top = hbm_roofline(dominant, avg_s(prof, dominant), model, pmc(dominant), ms_per_step,
                           prof[dominant]["launches"] / K, match)
    else:
        top = dict(gather, note=f"the largest share of the step is {dominant}, for which no byte model is kept")
    return top, gather, host_link


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
        enqueue_ms = None
        t0 = time.perf_counter()
        g.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        del g
    else:
        t0 = time.perf_counter()
        for e in range(W, W + K):
            lookups += b.step(e)
        t_enq = time.perf_counter()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        enqueue_ms = (t_enq - t0) * 1e3 / K
    assert b.s.sync_status() == 0
    ms_per_step = (t1 - t0) * 1e3 / K
    n_hit, n_miss = b.rm.n_hit_miss.cpu().tolist()
    n_staged = b.rm.n_unique_miss.cpu().tolist()[0] if b.coalesce else n_miss   # rows fetched over the link

    b.s.profile_enable(True)
    for e in range(W, W + K):
        b.step(e)
    prof = b.s.profile_read()
    b.s.profile_enable(False)
    if "stage_misses+small_sort" in prof:      # the fetch's launch also carried the backward pass's per-table sort
        prof["stage_misses"] = prof.pop("stage_misses+small_sort")
        prof["stage_misses"]["also_carries"] = "small_sort"
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
    b.s.set_tuning(binding.TUNE_PRESORT, b.presort_min_l if b.presort else 0)
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
    model = bytes_model(wl, L_avg, U, U_cold, n_miss, n_staged)
    if "pool_short_staged" in prof:
        # one index per bag, side-stream option: bags whose row is cached are pooled by one launch while the missed
        # rows are fetched, the others by a second launch after the fetch; the bytes split with the bags
        share = n_hit / max(1, n_hit + n_miss)
        whole = model["pool_short"]
        model["pool_short_staged"] = {k: v * (1 - share) for k, v in whole.items()}
        model["pool_short"] = {k: v * share for k, v in whole.items()}
    if "bwd_pairs" not in prof:    # the launch that lists hits and misses also wrote the backward pairs
        model["remap_write"] = {k: v + model["bwd_pairs"][k] for k, v in model["remap_write"].items()}
    kern = {}
    for name, r in prof.items():
        a_ms = r["total_ms"] / r["launches"]
        kern[name] = {"launches_per_step": r["launches"] / K, "avg_ms": round(a_ms, 5), "ms_per_step": round(r["total_ms"] / K, 5)}
        if name in model:
            kern[name]["alg_GBs"] = round(model[name]["alg"] / (a_ms * 1e-3) / 1e9, 1)
        if "also_carries" in r:
            kern[name]["also_carries"] = r["also_carries"]
    state_b = wl.dim * 4 if wl.optimizer == "adagrad" else 0
    # forward: every missed lookup's row is read over the link.  backward: a cold row's value comes from the copy
    # the forward pass staged, so only its accumulator is read over the link; row and accumulator are written back
    lb = {"fetch": n_staged * wl.row_bytes, "acc": U_cold * state_b, "write": U_cold * (wl.row_bytes + state_b)}
    link_bytes = lambda name: (lb["fetch"], 0) if name == "stage_misses" else (lb["acc"], lb["write"])
    top, gather, host_link = rooflines(wl, prof, K, ms_per_step, model, link, link_bytes, None, b.budget >= wl.total_rows * wl.row_bytes)
    if prof.get("stage_misses", {}).get("also_carries"):
        for r in [top] + host_link:
            if r.get("kernel") == "stage_misses":
                r["note"] = ("the first workgroups of this launch sort each table's (row, bag) pairs in LDS for the backward pass; "
                             "for a batch this small the sort, not the fetch, sets the launch's length, so the link figures "
                             "here are a lower bound on what the fetch reaches")
    pool = gather["kernel"]
    for tag, p in (("forward_alone", prof_fwd), ("forward_cold_caches", prof_cold)):
        t = avg_s(p, pool)
        gather[tag] = {"avg_launch_ms": round(t * 1e3, 5), "achieved": round(model[pool]["min"] / t / 1e9, 1),
                       "frac": round(min(1.0, model[pool]["min"] / t / 1e9 / HBM_PEAK_GBS), 4),
                       "effective_GBs": round(model[pool]["alg"] / t / 1e9, 1),
                       "effective_vs_peak": round(model[pool]["alg"] / t / 1e9 / HBM_PEAK_GBS, 4)}
        if gather.get("traffic"):
            gather[tag]["frac_counter"] = round(gather["traffic"] / t / 1e9 / HBM_PEAK_GBS, 4)
    return {"value": lookups / (t1 - t0), "ms_per_step": ms_per_step, "lookups_per_step": L_avg,
            "hit_rate": n_hit / max(1, n_hit + n_miss), "U": U, "U_cold": U_cold, "n_miss": n_miss, "n_staged": n_staged,
            "roofline": top, "gather": gather, "host_link": host_link, "kernels": kern,
            "calls_alone_ms": {c: round(v, 5) for c, v in alone.items()},
            "ms_per_step_median": round(per_step[len(per_step) // 2], 5), "ms_per_step_min": round(per_step[0], 5),
            "host_enqueue_ms_per_step": None if enqueue_ms is None else round(enqueue_ms, 5),
            "_model": model, "_pool": pool, "_link_bytes": lb}


def run_lookahead(b: Bench, K: int, W: int, leg: dict, link: dict) -> dict:
    """The same K batches in the look-ahead order: remap(e+1), update of batch e with the missed rows of batch e+1
    fetched beside it, forward pass of batch e+1.  Every batch still goes through remap, forward and update once,
    and every result is the one of the plain order (tests/test_gpu_lookahead.py)."""
    wl, s = b.wl, b.s
    n = len(b.batches)
    eps = wl.eps if wl.optimizer == "adagrad" else 0.0
    rms = [b.rm, s.new_remap_out()]
    s.set_tuning(binding.TUNE_LOOKAHEAD, 1)
    s.set_tuning(binding.TUNE_FUSED_FETCH, 1 if b.fused_fetch else 0)

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
    ms_per_step = (t1 - t0) * 1e3 / K
    timed0, serial0 = s.get_counter(binding.COUNTER_AHEAD_TIMED), s.get_counter(binding.COUNTER_AHEAD_NOT_OVERLAPPED)
    s.profile_enable(True)
    for e in range(W + K, W + 2 * K):
        step(e)
    prof = s.profile_read()
    s.profile_enable(False)
    timed = s.get_counter(binding.COUNTER_AHEAD_TIMED) - timed0
    serial = s.get_counter(binding.COUNTER_AHEAD_NOT_OVERLAPPED) - serial0
    s.set_tuning(binding.TUNE_LOOKAHEAD, 0)
    s.remap(*b.batches[0], wl.batch, b.rm)      # leave no look-ahead state behind for the legs that follow
    torch.cuda.synchronize()
    kern = {k: {"launches_per_step": v["launches"] / K, "avg_ms": round(v["total_ms"] / v["launches"], 5),
                "ms_per_step": round(v["total_ms"] / K, 5)} for k, v in prof.items()}
    # the link while the update runs: the fetch for the next batch and the accumulators come in, rows and
    # accumulators go out, at the same time (the few rows left to the forward pass's own fetch are not counted)
    lb = leg["_link_bytes"]
    fused = "seg_rows_long+fetch_ahead" in prof

    def link_bytes(name):
        if name == "stage_misses":
            return (0, 0)
        return (lb["acc"] + (lb["fetch"] if fused or "fetch_ahead" in prof else 0), lb["write"])

    top, gather, host_link = rooflines(wl, prof, K, ms_per_step, leg["_model"], link, link_bytes, leg["_pool"])
    return {"value": lookups / (t1 - t0), "unit": "lookups/s", "ms_per_step": ms_per_step,
            "forward_passes_with_rows_fetched_ahead": int(used), "steps": K,
            "fetch": "in the first workgroups of the update's own launch" if fused else "a launch of its own on the library's second stream",
            "updates_timed_beside_a_fetch_on_the_library_stream": int(timed), "of_which_not_overlapped": int(serial),
            "order": "remap(e+1) -> embedding_bag_bwd_update_ahead(e, e+1) -> embedding_bag_fwd(e+1)",
            "roofline": top, "gather": gather, "host_link": host_link, "kernels": kern}


def run_hot_normal(b: Bench, K: int, W: int, whole: dict) -> dict:
    """Section III of the paper trains samples whose lookups are all cached ("hot") and the others in mini-batches of
    their own.  One batch is classified and split on the device (scars_classify_samples, scars_partition_batch) and
    each sub-batch is run through remap, forward and update like any batch: the hot one touches no host memory."""
    wl, s = b.wl, b.s
    T = wl.num_tables
    idx, off = b.batches[0]
    s.remap(idx, off, wl.batch, b.rm)
    cls = s.classify_samples(idx, off, wl.batch, b.rm)
    n_hot, n_normal = cls.n_hot_normal.cpu().tolist()
    eps = wl.eps if wl.optimizer == "adagrad" else 0.0
    out = {"samples": wl.batch, "hot_samples": n_hot, "normal_samples": n_normal,
           "whole_batch": {"lookups_per_s": whole["value"], "ms_per_step": whole["ms_per_step"]}}
    subs = {}
    for name, ids, n, cnt in (("hot", cls.hot_ids, n_hot, cls.n_hot_normal[0:1]), ("normal", cls.normal_ids, n_normal, cls.n_hot_normal[1:2])):
        if n == 0:
            continue
        si, so, c = s.partition_batch(idx, off, wl.batch, ids, cnt)
        Ls, Gs = c.cpu().tolist()
        subs[name] = (si[:Ls].contiguous(), so[: T * n + 1].contiguous(), n, Ls)
    for name, (si, so, n, Ls) in subs.items():
        g = b.grads[0][: T * n].contiguous()
        o = b.out[: T * n]

        def step():
            s.remap(si, so, n, b.rm)
            s.embedding_bag_fwd(si, so, n, b.rm, o)
            s.embedding_bag_bwd_update(si, so, n, b.rm, g, wl.lr, eps)

        for _ in range(W):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(K):
            step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        n_hit, n_miss = b.rm.n_hit_miss.cpu().tolist()
        out[name] = {"samples": n, "lookups": Ls, "missed_lookups": n_miss, "lookups_per_s": Ls * K / (t1 - t0),
                     "ms_per_step": (t1 - t0) * 1e3 / K}
    assert s.sync_status() == 0
    if "hot" in out:
        assert out["hot"]["missed_lookups"] == 0
    if "hot" in out and "normal" in out:
        out["ms_hot_plus_normal"] = out["hot"]["ms_per_step"] + out["normal"]["ms_per_step"]
    return out


def cpu_baseline(b: Bench, seconds_target: float = 12.0) -> dict:
    """The CPU oracle, as it stands, on the machine's host cores, on a bounded sample of the same workload."""
    import oracle
    wl = b.wl
    cores = min(16, os.cpu_count() or 1)     # a one-GPU machine's CPU share is 16 cores, whatever os.cpu_count() shows
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
                      f"(report mode, nothing mutated) in {t_total:.1f}s.  A stated baseline, not a target: the oracle is "
                      f"the plain definition (fp64 sums, one qsort of the (row, position) pairs on a single thread, "
                      f"OpenMP only over bags and rows), so {used} threads gain little over one",
            "value_1_thread": one_L / one_t, "sample_1_thread": f"{one_nb} batch(es) in {one_t:.1f}s",
            "cpu_model": model, "host_cpus_visible": os.cpu_count()}


def measured_block(cal: dict, link: dict) -> dict:
    m = {"hbm_copy_GBs": round(cal["copy_GBs"], 1), "hbm_read_GBs": round(cal["read_GBs"], 1)}
    for k, v in link.items():
        m[k] = round(v, 2) if isinstance(v, float) else v
    return m


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="multi_hot", choices=synth.WORKLOAD_NAMES)
    ap.add_argument("--scale", type=float, default=1.0)
    ap.add_argument("--batch", type=int, default=0,
                    help="samples per table in a batch, for --workload only (default: the workload's own); the axis of the "
                         "paper's batch-size tables")
    ap.add_argument("--row-scale", type=float, default=None,
                    help="shrink table rows and budget only (default: 1.0, and for host_spill, whose 102 GB of tables "
                         "may exceed what the box lets one process pin, the largest multiple of 0.05 that can be pinned)")
    ap.add_argument("--budget-bytes", type=int, default=-1, help="override the workload's cache budget")
    ap.add_argument("--also", default="dlrm_onehot,low_skew,host_spill",
                    help="comma-separated other workloads to run briefly afterwards and report under other_workloads "
                         "('none' to skip)")
    ap.add_argument("--graph", action="store_true",
                    help="capture the K timed steps into one HIP graph and time its replay instead of K eager steps")
    ap.add_argument("--coalesce", action="store_true",
                    help="remap lists each distinct missed row once (Section II-A): one link read per unique cold row")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only-calibration", action="store_true",
                    help="measure the HBM and host-link ceilings (copy kernels, copies, scattered-piece kernels), print them and stop")
    ap.add_argument("--fused-long-max-l", type=int, default=-1,
                    help="largest batch (lookups) whose backward pass updates long runs and the other rows in one "
                         "launch (default: the library's, every batch; 0 = never)")
    ap.add_argument("--update-max-blocks", type=int, default=0,
                    help="most workgroups of the per-row update kernel (default: the library's, 8192)")
    ap.add_argument("--fused-scan-max-tiles", type=int, default=-1,
                    help="ordered compactions of up to this many 2048-item tiles add up the tile counts inside the "
                         "writing kernel instead of running a scan kernel between counting and writing (default: the library's)")
    ap.add_argument("--no-table-limit", dest="table_limit", action="store_false",
                    help="one-index-per-bag workloads: do not tell the library that a table gets at most `batch` lookups")
    ap.add_argument("--no-lookahead", dest="lookahead", action="store_false",
                    help="skip the extra leg in the look-ahead call order (reported under lookahead)")
    ap.add_argument("--fetch-on-own-stream", dest="fused_fetch", action="store_false",
                    help="look-ahead order: fetch the next batch's rows in a launch of its own on the library's second "
                         "stream instead of inside the update's launch")
    ap.add_argument("--presort-min-l", type=int, default=PRESORT_MIN_L,
                    help="smallest batch (lookups) whose backward sort is started on the library's side stream")
    ap.add_argument("--no-presort", dest="presort", action="store_false",
                    help="sort the backward pass's (row, bag) pairs inside bwd_update instead of starting that sort in "
                         "remap on the library's side stream, beside the forward pass")
    ap.set_defaults(presort=True, lookahead=True, fused_fetch=True, table_limit=True)
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
    if args.only_calibration:
        print(json.dumps({"measured": measured_block(cal, link)}), flush=True)
        return
    line = run_workload(args.workload, args, args.steps, args.warmup, cal, link, not args.no_cpu_baseline, args.resident)
    others = {}
    for name in [w for w in args.also.split(",") if w and w != "none" and w != args.workload]:
        # the other single-GPU workloads, shorter: parity-sized and link/latency-bound cases for context
        torch.cuda.empty_cache()
        r = run_workload(name, args, min(args.steps, 10), min(args.warmup, 3), cal, link, False, False)
        others[name] = {"value": r["value"], "unit": r["unit"], "ms_per_step": r["ms_per_step"], "dtype": r["dtype"],
                        "config": {k: r["config"][k] for k in ("row_scale", "scaled", "pinning", "rows", "dim", "batch", "lookups_per_step",
                                                                "hit_rate", "budget_bytes", "optimizer") if k in r["config"]},
                        "roofline": r["roofline"], "gather": r["gather"], "host_link": r["host_link"],
                        "call_order": r["config"]["step"].split("call order: ")[1],
                        "plain_order": {k: r["plain_order"][k] for k in ("value", "ms_per_step")},
                        "lookahead": r["lookahead"] and {k: r["lookahead"][k] for k in ("value", "ms_per_step")},
                        "build_cache_roofline": r["build_cache"]["roofline"], "hot_normal_split": r["hot_normal_split"]}
    line["other_workloads"] = others
    if args.also != "none" and args.workload != "low_skew_uniform":
        # the gather roofline reference: uniform ids over 6.4 GB of rows, every row cached (no reuse for the caches
        # to serve, so algorithmic bytes are close to HBM bytes)
        torch.cuda.empty_cache()
        r = run_workload("low_skew_uniform", args, min(args.steps, 10), min(args.warmup, 3), cal, link, False, False, True)
        line["gather_reference"] = {"workload": "low_skew_uniform, every row cached", "value": r["value"], "unit": r["unit"],
                                    "ms_per_step": r["ms_per_step"], "roofline": r["roofline"], "gather": r["gather"]}
    print(json.dumps(line), flush=True)


def run_workload(name: str, args, K: int, W: int, cal: dict, link: dict, with_cpu: bool, with_resident: bool,
                 all_cached: bool = False) -> dict:
    # host_spill asks for 102.4 GB of pinned tables: try that first, record what the box refuses, and step down
    forced = args.row_scale is not None
    row_scale = args.row_scale if forced else 1.0
    attempts = []
    while True:
        over = {"batch": args.batch} if (args.batch > 0 and name == args.workload) else {}
        wl = synth.workload(name, scale=args.scale, row_scale=row_scale, **over)
        pinned, failure = pin_tables(wl, wl.optimizer == "adagrad")
        if pinned is not None:
            break
        failure["row_scale"] = round(row_scale, 2)
        attempts.append(failure)
        log(name, "cannot pin its tables at row_scale", round(row_scale, 2), failure)
        if forced or row_scale <= 0.05 + 1e-9:
            raise SystemExit(f"bench.py: cannot pin the tables of {name}: {failure}")
        row_scale = round(row_scale - 0.05, 2)
    budget = wl.budget_bytes if (args.budget_bytes < 0 or name != args.workload) else args.budget_bytes
    if all_cached:
        budget = wl.total_rows * wl.row_bytes

    b = Bench(wl, budget, pinned, args.coalesce)
    b.presort = bool(args.presort)
    b.presort_min_l = args.presort_min_l
    if budget >= wl.total_rows * wl.row_bytes:
        b.presort_min_l = min(b.presort_min_l, PREPARE_MIN_L_CACHED)
    b.fused_fetch = bool(args.fused_fetch)
    b.s.set_tuning(binding.TUNE_PRESORT, b.presort_min_l if b.presort else 0)
    if args.fused_long_max_l >= 0:
        b.s.set_tuning(binding.TUNE_FUSED_LONG_MAX_L, args.fused_long_max_l)
    if args.update_max_blocks > 0:
        b.s.set_tuning(binding.TUNE_UPDATE_MAX_BLOCKS, args.update_max_blocks)
    if args.fused_scan_max_tiles >= 0:
        b.s.set_tuning(binding.TUNE_FUSED_SCAN_MAX_TILES, args.fused_scan_max_tiles)
    # one index per sample and table: a table gets exactly `batch` lookups, which the caller may state; up to 4096 the
    # backward pass then sorts each table's pairs in LDS (two launches instead of three per radix pass)
    table_limit = wl.batch if (wl.bag_lambda is None and args.table_limit) else 0
    b.s.set_tuning(binding.TUNE_MAX_TABLE_LOOKUPS, table_limit)
    b.prepare(K + W)
    bc = b.build_cache(link)
    log(name, "build_cache", bc)

    leg = run_leg(b, K, W, link, args.graph)
    ahead = None
    if args.lookahead and not args.coalesce:     # (with every row cached there is nothing to fetch ahead, but the next
        ahead = run_lookahead(b, K, W, leg, link)   #  batch's sort is still prepared beside this batch's update)
        log(name, "look-ahead order", {k: ahead[k] for k in ("value", "ms_per_step")})
    split = None
    if wl.bag_lambda is None and not args.coalesce and budget < wl.total_rows * wl.row_bytes:
        split = run_hot_normal(b, K, W, leg)      # one index per bag: a useful share of the samples is all-hot
        log(name, "hot / normal sub-batches", split)
    resident = None
    if with_resident and budget < wl.total_rows * wl.row_bytes and wl.total_rows * wl.row_bytes * 3 < 150e9:
        # second leg: every row cached (the paper's "hot" iteration): the same kernels, no host-link traffic
        b.s.flush_cache()
        torch.cuda.synchronize()
        b.budget = wl.total_rows * wl.row_bytes
        b.presort_min_l = min(b.presort_min_l, PREPARE_MIN_L_CACHED)
        b.s.set_tuning(binding.TUNE_PRESORT, b.presort_min_l if b.presort else 0)
        b.prepare(K + W)
        b.s.build_cache(None, None, 0, b.budget, 0)
        torch.cuda.synchronize()
        r = run_leg(b, K, W, link, args.graph)
        # ... and in the look-ahead order: nothing to fetch, but the next batch's sort and run starts are prepared on
        # the library's side stream while this batch's update (HBM-bound, several times as long) runs
        ra = run_lookahead(b, K, W, r, link) if (args.lookahead and not args.coalesce) else None
        best_r = ra if (ra is not None and ra["value"] > r["value"]) else r
        resident = {"value": best_r["value"], "unit": "lookups/s", "ms_per_step": best_r["ms_per_step"],
                    "order": best_r.get("order", "remap(e) -> embedding_bag_fwd(e) -> embedding_bag_bwd_update(e)"),
                    "plain_order": {"value": r["value"], "ms_per_step": r["ms_per_step"]},
                    "lookahead": ra and {"value": ra["value"], "ms_per_step": ra["ms_per_step"], "kernels": ra["kernels"]},
                    "ms_per_step_median": r["ms_per_step_median"], "ms_per_step_min": r["ms_per_step_min"],
                    "host_enqueue_ms_per_step": r["host_enqueue_ms_per_step"], "cached_rows": b.s.cache_rows(), "roofline": r["roofline"], "gather": r["gather"],
                    "calls_alone_ms": r["calls_alone_ms"], "kernels": r["kernels"],
                    "note": "roofline, gather, kernels, median and min are the plain order's"}
        log(name, "cache-resident leg", {k: resident[k] for k in ("value", "ms_per_step", "plain_order")})

    cpu = None
    b.s.flush_cache()           # host tables current again before the oracle reads them
    torch.cuda.synchronize()
    if with_cpu:
        cpu = cpu_baseline(b)
        log(name, "cpu_baseline", cpu)
    log(name, "lookups/s", f"{leg['value']:.4g}", "ms/step", f"{leg['ms_per_step']:.4f}")

    plain = {"value": leg["value"], "unit": "lookups/s", "ms_per_step": leg["ms_per_step"],
             "ms_per_step_median": leg["ms_per_step_median"], "ms_per_step_min": leg["ms_per_step_min"],
             "host_enqueue_ms_per_step": leg["host_enqueue_ms_per_step"],
             "order": "remap(e) -> embedding_bag_fwd(e) -> embedding_bag_bwd_update(e)",
             "roofline": leg["roofline"], "gather": leg["gather"], "host_link": leg["host_link"],
             "calls_alone_ms": leg["calls_alone_ms"], "kernels": leg["kernels"]}
    # the headline is the faster of the two call orders; both are reported in full (same batches, same results)
    best = ahead if (ahead is not None and ahead["value"] > leg["value"]) else plain
    gather = dict(best["gather"])
    if best is ahead:      # the gather kernel alone and with cold caches do not depend on the call order
        gather["forward_alone"] = leg["gather"]["forward_alone"]
        gather["forward_cold_caches"] = leg["gather"]["forward_cold_caches"]
    full_rows = synth.workload(name, scale=args.scale).total_rows
    line = {
        "metric": "pooled embedding lookups/sec (fwd+bwd) + achieved HBM GB/s, 1 GPU",
        "value": best["value"], "unit": "lookups/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": best["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if wl.dtype == "f32" else "bf16 storage, f32 sums", "data": "synthetic",
        "config": {"workload": wl.name, "scale": args.scale, "row_scale": row_scale, "scaled": wl.total_rows != full_rows,
                   "pinning": {"rows_of_the_full_workload": full_rows, "rows_run": wl.total_rows,
                               "refused_attempts": attempts,
                               "note": "full size" if wl.total_rows == full_rows else
                                       "the box refused to pin the full tables; this is the largest multiple of 0.05 of the rows it pins"},
                   "tables": wl.num_tables, "rows": wl.total_rows,
                   "dim": wl.dim, "batch": wl.batch, "lookups_per_step": leg["lookups_per_step"], "zipf_s": wl.zipf_s,
                   "budget_bytes": budget, "cached_rows": bc["k"], "optimizer": wl.optimizer,
                   "hit_rate": leg["hit_rate"], "unique_rows_per_step": leg["U"],
                   "unique_cold_rows_per_step": leg["U_cold"], "missed_lookups_per_step": leg["n_miss"],
                   "rows_fetched_over_link_per_step": leg["n_staged"], "coalesce": args.coalesce,
                   "launch": ("hip graph of the K steps" if args.graph else "eager") +
                             (", backward sort prepared on the library's side stream" if args.presort else "") +
                             (f", at most {table_limit} lookups per table stated (per-table sort in LDS)" if 0 < table_limit <= 4096 else ""),
                   "step": "every batch goes through remap, embedding_bag_fwd and embedding_bag_bwd_update once; call order: " + best["order"]},
        "roofline": best["roofline"], "gather": gather, "host_link": best["host_link"],
        "measured": measured_block(cal, link),
        "cpu_baseline": cpu, "cache_resident": resident, "plain_order": plain, "lookahead": ahead,
        "hot_normal_split": split,
        "kernels": best["kernels"], "build_cache": {k: (round(v, 4) if isinstance(v, float) else v) for k, v in bc.items()},
    }
    b.close()
    del b
    return line


if __name__ == "__main__":
    main()
