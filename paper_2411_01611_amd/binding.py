"""ctypes binding over libscars.so (the C ABI declared in include/scars.h).

Argument marshalling only: every step of the path runs in the library's HIP kernels.  PyTorch supplies
device memory (torch tensors whose data_ptr is handed over) and the current HIP stream.  There is no
fallback: if the library is missing or a call fails, this raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Dict, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# SCARS_LIB_PATH: load another build of the same sources instead (the test suite's host-sanitizer run sets it)
LIB_PATH = os.environ.get("SCARS_LIB_PATH") or os.path.join(_HERE, "libscars.so")

OK, ERR_INVALID_ARG, ERR_NOT_BUILT, ERR_WORKSPACE, ERR_HIP, ERR_INDEX_RANGE, ERR_OFFSETS = 0, -1, -2, -3, -4, -5, -6
DTYPE_F32, DTYPE_BF16 = 0, 1
OPT_SGD, OPT_ADAGRAD = 0, 1

EXPORTS = (
    "scars_create", "scars_destroy", "scars_set_tuning", "scars_get_counter", "scars_query_sizes", "scars_bind_buffers", "scars_build_cache",
    "scars_cache_rows", "scars_remap", "scars_remap_static", "scars_classify_samples", "scars_partition_batch", "scars_portion_usage", "scars_epoch_cost",
    "scars_caching_gain",
    "scars_plan_cache", "scars_embedding_bag_fwd", "scars_embedding_bag_bwd_update", "scars_embedding_bag_bwd_update_ahead",
    "scars_flush_cache", "scars_sync_status", "scars_last_error", "scars_host_alloc", "scars_host_free",
    "scars_memcpy", "scars_calibration_copy", "scars_calibration_read", "scars_calibration_link", "scars_profile_enable", "scars_profile_read",
)


class ScarsError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"scars error {code}: {msg}")
        self.code = code


class _Config(C.Structure):
    _fields_ = [("num_tables", C.c_int32), ("rows", C.POINTER(C.c_int64)), ("dim", C.c_int32), ("dtype", C.c_int32),
                ("host_tables", C.POINTER(C.c_void_p)), ("optimizer", C.c_int32), ("host_state", C.POINTER(C.c_void_p))]


class _Sizes(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("k", "counts_bytes", "slot_of_bytes", "hot_gid_bytes", "cache_bytes",
                                         "state_cache_bytes", "workspace_bytes", "per_lookup_bytes",
                                         "seg_start_bytes", "out_bytes")]


class _Buffers(C.Structure):
    _fields_ = [("counts", C.c_void_p), ("slot_of", C.c_void_p), ("hot_gid", C.c_void_p), ("cache", C.c_void_p),
                ("state_cache", C.c_void_p), ("workspace", C.c_void_p), ("budget_bytes", C.c_int64),
                ("max_L", C.c_int64), ("max_G", C.c_int64), ("counts_bytes", C.c_int64), ("slot_of_bytes", C.c_int64),
                ("hot_gid_bytes", C.c_int64), ("cache_bytes", C.c_int64), ("state_cache_bytes", C.c_int64),
                ("workspace_bytes", C.c_int64)]


class _RemapOut(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("slot", "gid", "loc", "hit_pos", "miss_pos", "miss_gid", "n_hit_miss",
                                          "unique_miss_gid", "n_unique_miss")]


class _BwdOut(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("sorted_gid", "sorted_bag", "seg_start", "unique_gid", "n_unique")]


class _ClassifyOut(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("is_hot", "hot_ids", "normal_ids", "n_hot_normal")]


class _SubbatchOut(C.Structure):
    _fields_ = [("indices", C.c_void_p), ("offsets", C.c_void_p), ("n_lookups_bags", C.c_void_p)]


class _PlanIn(C.Structure):
    _fields_ = [("device_params", C.c_double), ("per_sample_params", C.c_double), ("samples_per_epoch", C.c_double),
                ("profile_samples", C.c_int64)]


class _PlanOut(C.Structure):
    _fields_ = [("best_k", C.c_int64), ("best_cost", C.c_double), ("best_batch", C.c_double), ("cost_no_cache", C.c_double),
                ("batch_no_cache", C.c_double), ("k_max", C.c_int64)]


class _KernelTime(C.Structure):
    _fields_ = [("name", C.c_char_p), ("launches", C.c_int64), ("total_ms", C.c_double)]


_lib = None


def lib():
    """Load libscars.so; fails loudly when it has not been built (no CPU fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2411_01611_amd.build`")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
        L.scars_create.argtypes = [C.POINTER(_Config), C.POINTER(vp)]
        L.scars_destroy.argtypes = [vp]
        L.scars_set_tuning.argtypes = [vp, i32, i64]
        L.scars_get_counter.argtypes = [vp, i32]
        L.scars_get_counter.restype = i64
        L.scars_query_sizes.argtypes = [vp, i64, i64, i64, C.POINTER(_Sizes)]
        L.scars_bind_buffers.argtypes = [vp, C.POINTER(_Buffers), vp]
        L.scars_build_cache.argtypes = [vp, vp, vp, i64, i64, i64, i32, vp]
        L.scars_cache_rows.argtypes = [vp]
        L.scars_cache_rows.restype = i64
        L.scars_remap.argtypes = [vp, vp, vp, i64, i64, C.POINTER(_RemapOut), vp]
        L.scars_remap_static.argtypes = [vp, vp, vp, i64, i64, C.POINTER(_RemapOut), vp]
        L.scars_embedding_bag_fwd.argtypes = [vp, vp, vp, i64, i64, C.POINTER(_RemapOut), vp, vp]
        L.scars_embedding_bag_bwd_update.argtypes = [vp, vp, vp, i64, i64, C.POINTER(_RemapOut), vp, f32, f32,
                                                     C.POINTER(_BwdOut), vp]
        L.scars_embedding_bag_bwd_update_ahead.argtypes = [vp, vp, vp, i64, i64, C.POINTER(_RemapOut), vp, f32, f32,
                                                           C.POINTER(_BwdOut), C.POINTER(_RemapOut), vp, i64, i64, vp]
        L.scars_classify_samples.argtypes = [vp, vp, i64, i64, C.POINTER(_RemapOut), C.POINTER(_ClassifyOut), vp]
        L.scars_partition_batch.argtypes = [vp, vp, vp, i64, i64, vp, vp, C.POINTER(_SubbatchOut), vp]
        L.scars_portion_usage.argtypes = [vp, vp, i64, i64, C.POINTER(_RemapOut), i64, i32, vp, vp]
        L.scars_epoch_cost.argtypes = [vp, C.POINTER(_PlanIn), i64, C.POINTER(C.c_double), C.POINTER(C.c_double), vp]
        L.scars_caching_gain.argtypes = [vp, C.POINTER(_PlanIn), i64, C.POINTER(C.c_double), C.POINTER(C.c_double), vp]
        L.scars_plan_cache.argtypes = [vp, C.POINTER(_PlanIn), C.POINTER(_PlanOut), vp]
        L.scars_flush_cache.argtypes = [vp, vp]
        L.scars_sync_status.argtypes = [vp, vp]
        L.scars_last_error.argtypes = [vp]
        L.scars_last_error.restype = C.c_char_p
        L.scars_host_alloc.argtypes = [i64, C.POINTER(vp)]
        L.scars_host_free.argtypes = [vp]
        L.scars_memcpy.argtypes = [vp, vp, i64, i32, vp]
        L.scars_calibration_copy.argtypes = [vp, vp, i64, vp]
        L.scars_calibration_read.argtypes = [vp, i64, vp, vp]
        L.scars_calibration_link.argtypes = [vp, i64, vp, i64, i32, i32, i32, i32, vp]
        L.scars_profile_enable.argtypes = [vp, i32]
        L.scars_profile_read.argtypes = [vp, vp, C.POINTER(_KernelTime), i32, C.POINTER(i32)]
        _lib = L
    return _lib


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


CALIB_SINK_BYTES = 4 << 20
TUNE_FUSED_SCAN_MAX_TILES, TUNE_PRESORT, TUNE_FUSED_LONG_MAX_L, TUNE_PAIRS_IN_REMAP, TUNE_UPDATE_MAX_BLOCKS = 1, 2, 3, 4, 5
TUNE_LOOKAHEAD = 6
TUNE_FUSED_FETCH = 7
TUNE_MAX_TABLE_LOOKUPS = 8
COUNTER_PREPARED_USED = 1
COUNTER_AHEAD_USED = 2
COUNTER_AHEAD_TIMED = 3
COUNTER_AHEAD_NOT_OVERLAPPED = 4
COUNTER_SORTED_IN_FWD_USED = 5


def calibration_read(src: torch.Tensor, sink: torch.Tensor) -> None:
    """Launch the plain read-only kernel on the current stream (sink: CUDA tensor of at least CALIB_SINK_BYTES)."""
    n = src.numel() * src.element_size()
    assert n % 16 == 0 and sink.numel() * sink.element_size() >= CALIB_SINK_BYTES
    rc = lib().scars_calibration_read(src.data_ptr(), n, sink.data_ptr(), _stream())
    if rc != OK:
        raise ScarsError(rc, "calibration read failed")


def calibration_link(host: "PinnedArray", dev: torch.Tensor, n_granules: int, granule_bytes: int, scattered: bool,
                     to_host: bool, workgroups: int = 128) -> None:
    """Launch the host-link calibration kernel on the current stream (see scars_calibration_link)."""
    assert dev.is_cuda and dev.numel() * dev.element_size() >= n_granules * granule_bytes
    rc = lib().scars_calibration_link(host.ptr, host.nbytes, dev.data_ptr(), n_granules, granule_bytes, int(scattered),
                                      int(to_host), workgroups, _stream())
    if rc != OK:
        raise ScarsError(rc, "link calibration failed")


def calibration_copy(dst: torch.Tensor, src: torch.Tensor) -> None:
    """Launch the plain copy kernel on the current stream (dst, src: contiguous CUDA tensors of equal byte size)."""
    n = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == n and n % 16 == 0
    rc = lib().scars_calibration_copy(dst.data_ptr(), src.data_ptr(), n, _stream())
    if rc != OK:
        raise ScarsError(rc, "calibration copy failed")


def memcpy(dst_ptr: int, src_ptr: int, nbytes: int, kind: int) -> None:
    """hipMemcpyAsync on the current stream; kind 1 = host-to-device, 2 = device-to-host, 3 = device-to-device."""
    rc = lib().scars_memcpy(dst_ptr, src_ptr, nbytes, kind, _stream())
    if rc != OK:
        raise ScarsError(rc, "memcpy failed")


class PinnedArray:
    """Host memory from hipHostMalloc (device-mapped), viewed as a numpy array / CPU torch tensor."""

    def __init__(self, shape, dtype: np.dtype):
        self.shape = tuple(int(s) for s in shape)
        self.dtype = np.dtype(dtype)
        self.nbytes = int(np.prod(self.shape)) * self.dtype.itemsize
        p = C.c_void_p()
        rc = lib().scars_host_alloc(max(self.nbytes, 16), C.byref(p))
        if rc != OK:
            raise ScarsError(rc, f"hipHostMalloc of {self.nbytes} bytes failed")
        self.ptr = p.value
        buf = (C.c_char * max(self.nbytes, 1)).from_address(self.ptr)
        self.np = np.frombuffer(buf, dtype=self.dtype, count=int(np.prod(self.shape))).reshape(self.shape)

    def torch(self) -> torch.Tensor:
        return torch.from_numpy(self.np)

    def copy_from_device(self, src: torch.Tensor, row0: int = 0) -> None:
        """Asynchronous device-to-pinned copy of `src` into rows [row0, row0 + len(src)) on the current stream."""
        assert src.is_cuda and src.is_contiguous()
        nbytes = src.numel() * src.element_size()
        off = row0 * (self.nbytes // self.shape[0]) if self.shape[0] else 0
        rc = lib().scars_memcpy(self.ptr + off, src.data_ptr(), nbytes, 2, _stream())
        if rc != OK:
            raise ScarsError(rc, "device-to-host copy failed")

    def free(self) -> None:
        if self.ptr:
            self.np = None
            lib().scars_host_free(self.ptr)
            self.ptr = 0

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


@dataclass
class RemapOut:
    slot: torch.Tensor
    gid: torch.Tensor
    loc: torch.Tensor
    hit_pos: torch.Tensor
    miss_pos: torch.Tensor
    miss_gid: torch.Tensor
    n_hit_miss: torch.Tensor
    unique_miss_gid: Optional[torch.Tensor] = None     # set both to have remap coalesce the missed rows
    n_unique_miss: Optional[torch.Tensor] = None

    def c(self) -> _RemapOut:
        opt = lambda t: t.data_ptr() if t is not None else None
        return _RemapOut(*[t.data_ptr() for t in (self.slot, self.gid, self.loc, self.hit_pos, self.miss_pos,
                                                  self.miss_gid, self.n_hit_miss)],
                         opt(self.unique_miss_gid), opt(self.n_unique_miss))


@dataclass
class BwdOut:
    sorted_gid: torch.Tensor
    sorted_bag: torch.Tensor
    seg_start: torch.Tensor
    unique_gid: torch.Tensor
    n_unique: torch.Tensor

    def c(self) -> _BwdOut:
        return _BwdOut(*[t.data_ptr() for t in (self.sorted_gid, self.sorted_bag, self.seg_start, self.unique_gid,
                                                self.n_unique)])


@dataclass
class ClassifyOut:
    is_hot: torch.Tensor
    hot_ids: torch.Tensor
    normal_ids: torch.Tensor
    n_hot_normal: torch.Tensor

    def c(self) -> _ClassifyOut:
        return _ClassifyOut(*[t.data_ptr() for t in (self.is_hot, self.hot_ids, self.normal_ids, self.n_hot_normal)])


class Scars:
    """One handle: tables in pinned host memory, caller-side device buffers, the four calls."""

    def __init__(self, rows: Sequence[int], dim: int, dtype: int, host_table_ptrs: Sequence[int], optimizer: int = OPT_SGD,
                 host_state_ptrs: Optional[Sequence[int]] = None):
        self._h = C.c_void_p()
        self.rows = [int(r) for r in rows]
        self.T, self.D, self.dtype, self.optimizer = len(self.rows), int(dim), int(dtype), int(optimizer)
        self.N = sum(self.rows)
        self.R = self.D * (4 if dtype == DTYPE_F32 else 2)
        rows_a = (C.c_int64 * self.T)(*self.rows)
        tabs = (C.c_void_p * self.T)(*[int(p) for p in host_table_ptrs])
        st = (C.c_void_p * self.T)(*[int(p) for p in host_state_ptrs]) if host_state_ptrs is not None else None
        cfg = _Config(self.T, rows_a, self.D, self.dtype, tabs, self.optimizer, st)
        rc = lib().scars_create(C.byref(cfg), C.byref(self._h))
        if rc != OK:
            self._h = C.c_void_p()
            raise ScarsError(rc, "scars_create rejected the configuration")
        self.bufs: Dict[str, torch.Tensor] = {}
        self.max_L = self.max_G = 0
        self.budget_bytes = 0

    # ---- plumbing -----------------------------------------------------------------------------------
    def _check(self, rc: int) -> None:
        if rc != OK:
            raise ScarsError(rc, lib().scars_last_error(self._h).decode())

    def close(self) -> None:
        if self._h:
            lib().scars_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def query_sizes(self, budget_bytes: int, max_L: int, max_G: int) -> Dict[str, int]:
        s = _Sizes()
        self._check(lib().scars_query_sizes(self._h, budget_bytes, max_L, max_G, C.byref(s)))
        return {n: int(getattr(s, n)) for n, _ in _Sizes._fields_}

    def bind_buffers(self, budget_bytes: int, max_L: int, max_G: int, device="cuda:0") -> Dict[str, int]:
        """Allocate the device buffers scars_query_sizes asks for (as torch tensors) and bind them."""
        sz = self.query_sizes(budget_bytes, max_L, max_G)
        dev = torch.device(device)
        mk = lambda nbytes: torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
        self.bufs = {n: mk(sz[n + "_bytes"]) for n in ("counts", "slot_of", "hot_gid", "cache", "workspace")}
        self.bufs["state_cache"] = mk(sz["state_cache_bytes"]) if self.optimizer == OPT_ADAGRAD else None
        b = _Buffers(self.bufs["counts"].data_ptr(), self.bufs["slot_of"].data_ptr(), self.bufs["hot_gid"].data_ptr(),
                     self.bufs["cache"].data_ptr(),
                     self.bufs["state_cache"].data_ptr() if self.bufs["state_cache"] is not None else None,
                     self.bufs["workspace"].data_ptr(), budget_bytes, max_L, max_G,
                     *[self.bufs[n].numel() if self.bufs[n] is not None else 0
                       for n in ("counts", "slot_of", "hot_gid", "cache", "state_cache", "workspace")])
        self._check(lib().scars_bind_buffers(self._h, C.byref(b), _stream()))
        self.max_L, self.max_G, self.budget_bytes, self.device = max_L, max_G, budget_bytes, dev
        return sz

    def new_remap_out(self, L: Optional[int] = None, coalesce: bool = False) -> RemapOut:
        n = max(self.max_L if L is None else L, 1)
        mk = lambda m: torch.empty(m, dtype=torch.int32, device=self.device)
        return RemapOut(mk(n), mk(n), mk(n), mk(n), mk(n), mk(n), mk(2), mk(n) if coalesce else None,
                        mk(2) if coalesce else None)

    def new_bwd_out(self, L: Optional[int] = None) -> BwdOut:
        n = max(self.max_L if L is None else L, 1)
        mk = lambda m: torch.empty(m, dtype=torch.int32, device=self.device)
        return BwdOut(mk(n), mk(n), mk(n + 1), mk(n), mk(2))

    # views of the bound buffers
    def counts(self) -> torch.Tensor:
        return self.bufs["counts"][: self.N * 4].view(torch.int32)

    def slot_of(self) -> torch.Tensor:
        return self.bufs["slot_of"][: self.N * 4].view(torch.int32)

    def hot_gid(self) -> torch.Tensor:
        k = self.cache_rows()
        return self.bufs["hot_gid"][: k * 4].view(torch.int32)

    def cache(self) -> torch.Tensor:
        k = self.cache_rows()
        dt = torch.float32 if self.dtype == DTYPE_F32 else torch.bfloat16
        return self.bufs["cache"][: k * self.R].view(dt).view(k, self.D)

    def state_cache(self) -> torch.Tensor:
        k = self.cache_rows()
        return self.bufs["state_cache"][: k * self.D * 4].view(torch.float32).view(k, self.D)

    # ---- the calls ----------------------------------------------------------------------------------
    @staticmethod
    def _i32(t: Optional[torch.Tensor]):
        if t is None:
            return None
        assert t.is_cuda and t.dtype == torch.int32 and t.is_contiguous()
        return t.data_ptr()

    def build_cache(self, indices: Optional[torch.Tensor], offsets: Optional[torch.Tensor], bags_per_table: int,
                    budget_bytes: int, accumulate: int = 0) -> None:
        Lp = int(indices.numel()) if indices is not None else 0
        self._check(lib().scars_build_cache(self._h, self._i32(indices), self._i32(offsets), Lp, bags_per_table,
                                            budget_bytes, accumulate, _stream()))

    def cache_rows(self) -> int:
        return int(lib().scars_cache_rows(self._h))

    def remap(self, indices: torch.Tensor, offsets: torch.Tensor, B: int, out: Optional[RemapOut] = None,
              coalesce: bool = False) -> RemapOut:
        L = int(indices.numel())
        out = out or self.new_remap_out(L, coalesce)
        c = out.c()
        self._check(lib().scars_remap(self._h, self._i32(indices), self._i32(offsets), L, B, C.byref(c), _stream()))
        return out

    def remap_static(self, indices: torch.Tensor, offsets: torch.Tensor, B: int, out: RemapOut) -> RemapOut:
        """scars_remap_static: the remap whose scratch is the library's static device array (allocates nothing, so the
        output arrays must be passed in)."""
        c = out.c()
        self._check(lib().scars_remap_static(self._h, self._i32(indices), self._i32(offsets), int(indices.numel()), B,
                                             C.byref(c), _stream()))
        return out

    def embedding_bag_fwd(self, indices: torch.Tensor, offsets: torch.Tensor, B: int, rm: RemapOut,
                          out: Optional[torch.Tensor] = None) -> torch.Tensor:
        L = int(indices.numel())
        if out is None:
            out = torch.empty(self.T * B, self.D, dtype=torch.float32, device=self.device)
        assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous() and out.numel() == self.T * B * self.D
        c = rm.c()
        self._check(lib().scars_embedding_bag_fwd(self._h, self._i32(indices), self._i32(offsets), L, B, C.byref(c),
                                                  out.data_ptr(), _stream()))
        return out

    def embedding_bag_bwd_update(self, indices: torch.Tensor, offsets: torch.Tensor, B: int, rm: RemapOut,
                                 grad_out: torch.Tensor, lr: float, eps: float = 0.0,
                                 out: Optional[BwdOut] = None) -> Optional[BwdOut]:
        L = int(indices.numel())
        assert grad_out.is_cuda and grad_out.dtype == torch.float32 and grad_out.is_contiguous()
        assert grad_out.numel() == self.T * B * self.D
        c = rm.c()
        co = out.c() if out is not None else None
        self._check(lib().scars_embedding_bag_bwd_update(self._h, self._i32(indices), self._i32(offsets), L, B,
                                                         C.byref(c), grad_out.data_ptr(), lr, eps,
                                                         C.byref(co) if co is not None else None, _stream()))
        return out

    def embedding_bag_bwd_update_ahead(self, indices: torch.Tensor, offsets: torch.Tensor, B: int, rm: RemapOut,
                                       grad_out: torch.Tensor, lr: float, eps: float, next_rm: RemapOut,
                                       next_indices: torch.Tensor, next_offsets: torch.Tensor, next_B: int,
                                       out: Optional[BwdOut] = None) -> Optional[BwdOut]:
        """The update of this batch, with the next batch's missed rows fetched beside it (TUNE_LOOKAHEAD must be on)."""
        L = int(indices.numel())
        assert grad_out.is_cuda and grad_out.dtype == torch.float32 and grad_out.is_contiguous()
        assert grad_out.numel() == self.T * B * self.D
        c, cn = rm.c(), next_rm.c()
        co = out.c() if out is not None else None
        self._check(lib().scars_embedding_bag_bwd_update_ahead(self._h, self._i32(indices), self._i32(offsets), L, B,
                                                               C.byref(c), grad_out.data_ptr(), lr, eps,
                                                               C.byref(co) if co is not None else None, C.byref(cn),
                                                               self._i32(next_offsets), int(next_indices.numel()), next_B,
                                                               _stream()))
        return out

    def classify_samples(self, indices: torch.Tensor, offsets: torch.Tensor, B: int, rm: RemapOut,
                         out: Optional[ClassifyOut] = None) -> ClassifyOut:
        if out is None:
            mk = lambda m: torch.empty(max(m, 1), dtype=torch.int32, device=self.device)
            out = ClassifyOut(mk(B), mk(B), mk(B), mk(2))
        c, co = rm.c(), out.c()
        self._check(lib().scars_classify_samples(self._h, self._i32(offsets), int(indices.numel()), B, C.byref(c),
                                                 C.byref(co), _stream()))
        return out

    def partition_batch(self, indices: torch.Tensor, offsets: torch.Tensor, B: int, ids: torch.Tensor, n: torch.Tensor):
        """Sub-batch of the samples ids[:n] (n: 1-element int32 CUDA tensor, e.g. cls.n_hot_normal[0:1]).
        Returns (sub_indices [L], sub_offsets [T*B+1], n_lookups_bags [2]); only the leading parts are valid."""
        L = int(indices.numel())
        sub_idx = torch.empty(max(L, 1), dtype=torch.int32, device=self.device)
        sub_off = torch.empty(self.T * B + 1, dtype=torch.int32, device=self.device)
        cnt = torch.zeros(2, dtype=torch.int32, device=self.device)
        assert ids.is_cuda and ids.dtype == torch.int32 and n.is_cuda and n.dtype == torch.int32
        c = _SubbatchOut(sub_idx.data_ptr(), sub_off.data_ptr(), cnt.data_ptr())
        self._check(lib().scars_partition_batch(self._h, self._i32(indices), self._i32(offsets), L, B, ids.data_ptr(),
                                                n.data_ptr(), C.byref(c), _stream()))
        return sub_idx, sub_off, cnt

    def portion_usage(self, indices: torch.Tensor, offsets: torch.Tensor, B: int, rm: RemapOut, portion_rows: int,
                      n_portions: int) -> torch.Tensor:
        usage = torch.empty(n_portions, dtype=torch.int32, device=self.device)
        c = rm.c()
        self._check(lib().scars_portion_usage(self._h, self._i32(offsets), int(indices.numel()), B, C.byref(c),
                                              portion_rows, n_portions, usage.data_ptr(), _stream()))
        return usage

    def set_tuning(self, which: int, value: int) -> None:
        self._check(lib().scars_set_tuning(self._h, which, value))

    def get_counter(self, which: int) -> int:
        return int(lib().scars_get_counter(self._h, which))

    def epoch_cost(self, M: float, a: float, Q: float, profile_samples: int, k: int):
        """(cost, batch size) of eq. (6)/(7) for k cached rows, from the skew table now on the device.  Blocks."""
        pin = _PlanIn(M, a, Q, profile_samples)
        cost, b = C.c_double(0.0), C.c_double(0.0)
        self._check(lib().scars_epoch_cost(self._h, C.byref(pin), k, C.byref(cost), C.byref(b), _stream()))
        return cost.value, b.value

    def caching_gain(self, M: float, a: float, profile_samples: int, k: int):
        """(lhs, t1) of eq. (11)/(12) for caching the row ranked k + 1 on top of the first k.  Blocks."""
        pin = _PlanIn(M, a, 1.0, profile_samples)
        lhs, t1 = C.c_double(0.0), C.c_double(0.0)
        self._check(lib().scars_caching_gain(self._h, C.byref(pin), k, C.byref(lhs), C.byref(t1), _stream()))
        return lhs.value, t1.value

    def plan_cache(self, M: float, a: float, Q: float, profile_samples: int) -> Dict[str, float]:
        pin, po = _PlanIn(M, a, Q, profile_samples), _PlanOut()
        self._check(lib().scars_plan_cache(self._h, C.byref(pin), C.byref(po), _stream()))
        return {n: getattr(po, n) for n, _ in _PlanOut._fields_}

    def flush_cache(self) -> None:
        self._check(lib().scars_flush_cache(self._h, _stream()))

    def sync_status(self) -> int:
        """Blocks; returns the latched device-side error code (0 if none) and clears it."""
        return int(lib().scars_sync_status(self._h, _stream()))

    def profile_enable(self, on: bool) -> None:
        self._check(lib().scars_profile_enable(self._h, 1 if on else 0))

    def profile_read(self) -> Dict[str, Dict[str, float]]:
        arr = (_KernelTime * 64)()
        n = C.c_int32(0)
        self._check(lib().scars_profile_read(self._h, _stream(), arr, 64, C.byref(n)))
        return {arr[i].name.decode(): {"launches": int(arr[i].launches), "total_ms": float(arr[i].total_ms)}
                for i in range(n.value)}
