"""ctypes loader for the CPU oracle -- TEST INFRASTRUCTURE ONLY.

Only `tests/`, the smoke check and the benchmark's cpu_baseline leg import this package; the
product path never does.  Arguments are numpy arrays (host memory); every call is synchronous.
`build()` compiles `scars_oracle.c` with gcc into `liboracle.so` beside it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# SCARS_ORACLE_SO: load another build of scars_oracle.c instead (the test suite's sanitizer run sets it)
_SO = os.environ.get("SCARS_ORACLE_SO") or os.path.join(_HERE, "liboracle.so")
_lib = None

OK, ERR_INVALID_ARG, ERR_INDEX_RANGE, ERR_OFFSETS = 0, -1, -5, -6


def build(force: bool = True) -> str:
    src = os.path.join(_HERE, "scars_oracle.c")
    if os.environ.get("SCARS_ORACLE_SO"):
        return _SO
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", _SO, src, "-lm"])
    return _SO


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            build()
        _lib = C.CDLL(_SO)
        _lib.ora_budget_rows.restype = C.c_int64
        _lib.ora_budget_rows.argtypes = [C.c_int64] * 3
    return _lib


def _p(a: Optional[np.ndarray]):
    if a is None:
        return None
    assert a.flags["C_CONTIGUOUS"]
    return C.c_void_p(a.ctypes.data)


def _rows(rows: Sequence[int]) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(rows, dtype=np.int64))


def _ptr_array(arrs: Sequence[np.ndarray]):
    for a in arrs:
        assert a.flags["C_CONTIGUOUS"]
    return (C.c_void_p * len(arrs))(*[a.ctypes.data for a in arrs])


def _i32(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.int32
    return a


def set_threads(n: int) -> int:
    return int(lib().ora_set_threads(C.c_int32(n)))


def budget_rows(n_rows: int, row_bytes: int, budget_bytes: int) -> int:
    return int(lib().ora_budget_rows(n_rows, row_bytes, budget_bytes))


def _LB(rows, offsets, B):
    T = len(rows)
    assert offsets.shape[0] == T * B + 1
    return T


def histogram(rows, indices, offsets, B: int, counts: Optional[np.ndarray] = None) -> Tuple[int, np.ndarray]:
    rows = _rows(rows); indices = _i32(indices); offsets = _i32(offsets)
    T = _LB(rows, offsets, B)
    if counts is None:
        counts = np.zeros(int(rows.sum()), dtype=np.uint32)
    rc = lib().ora_histogram(C.c_int32(T), _p(rows), _p(indices), _p(offsets), C.c_int64(indices.shape[0]),
                             C.c_int64(B), _p(counts))
    return rc, counts


def hot_set(counts: np.ndarray, k: int) -> Tuple[int, np.ndarray, np.ndarray]:
    counts = np.ascontiguousarray(counts, dtype=np.uint32)
    N = counts.shape[0]
    hot = np.empty(max(k, 0), dtype=np.int32)
    slot_of = np.empty(N, dtype=np.int32)
    rc = lib().ora_hot_set(C.c_int64(N), _p(counts), C.c_int64(k), _p(hot), _p(slot_of))
    return rc, hot, slot_of


def remap(rows, indices, offsets, B: int, slot_of: np.ndarray):
    rows = _rows(rows); indices = _i32(indices); offsets = _i32(offsets); slot_of = _i32(slot_of)
    T = _LB(rows, offsets, B)
    L = indices.shape[0]
    slot = np.full(L, -7, dtype=np.int32)
    hit = np.empty(L, dtype=np.int32); miss = np.empty(L, dtype=np.int32); mg = np.empty(L, dtype=np.int32)
    n = np.zeros(2, dtype=np.int64)
    rc = lib().ora_remap(C.c_int32(T), _p(rows), _p(indices), _p(offsets), C.c_int64(L), C.c_int64(B),
                         _p(slot_of), _p(slot), _p(hit), _p(miss), _p(mg), _p(n))
    if rc in (OK, ERR_INDEX_RANGE):
        return rc, slot, hit[: n[0]].copy(), miss[: n[1]].copy(), mg[: n[1]].copy()
    return rc, None, None, None, None


def coalesce(miss_gid: np.ndarray):
    miss_gid = _i32(miss_gid)
    n = miss_gid.shape[0]
    uq = np.empty(max(n, 1), dtype=np.int32); inv = np.empty(max(n, 1), dtype=np.int32)
    U = np.zeros(1, dtype=np.int64)
    rc = lib().ora_coalesce(C.c_int64(n), _p(miss_gid), _p(uq), _p(inv), _p(U))
    return rc, uq[: int(U[0])].copy(), inv[:n].copy()


def classify_samples(rows, indices, offsets, B: int, slot_of: np.ndarray):
    rows = _rows(rows); indices = _i32(indices); offsets = _i32(offsets); slot_of = _i32(slot_of)
    T = _LB(rows, offsets, B)
    is_hot = np.empty(max(B, 1), dtype=np.int32); hot = np.empty(max(B, 1), dtype=np.int32)
    normal = np.empty(max(B, 1), dtype=np.int32)
    n = np.zeros(2, dtype=np.int64)
    rc = lib().ora_classify_samples(C.c_int32(T), _p(rows), _p(indices), _p(offsets), C.c_int64(indices.shape[0]),
                                    C.c_int64(B), _p(slot_of), _p(is_hot), _p(hot), _p(normal), _p(n))
    if rc in (OK, ERR_INDEX_RANGE):
        return rc, is_hot[:B].copy(), hot[: n[0]].copy(), normal[: n[1]].copy()
    return rc, None, None, None


def partition_batch(T: int, indices, offsets, B: int, ids):
    """Sub-batch of the samples `ids` (ascending): (rc, sub_indices, sub_offsets)."""
    indices = _i32(indices); offsets = _i32(offsets); ids = _i32(ids)
    L, n = indices.shape[0], ids.shape[0]
    sub_idx = np.empty(max(L, 1), dtype=np.int32)
    sub_off = np.empty(T * n + 1, dtype=np.int32)
    Ls = C.c_int64(0)
    rc = lib().ora_partition_batch(C.c_int32(T), _p(indices), _p(offsets), C.c_int64(L), C.c_int64(B), _p(ids),
                                   C.c_int64(n), _p(sub_idx), _p(sub_off), C.byref(Ls))
    return rc, sub_idx[: Ls.value], sub_off


def portion_usage(rows, indices, offsets, B: int, slot_of: np.ndarray, portion_rows: int, n_portions: int):
    rows = _rows(rows); indices = _i32(indices); offsets = _i32(offsets); slot_of = _i32(slot_of)
    T = _LB(rows, offsets, B)
    usage = np.zeros(n_portions, dtype=np.int32)
    rc = lib().ora_portion_usage(C.c_int32(T), _p(rows), _p(indices), _p(offsets), C.c_int64(indices.shape[0]),
                                 C.c_int64(B), _p(slot_of), C.c_int64(portion_rows), C.c_int32(n_portions), _p(usage))
    return rc, usage


def epoch_cost(T: int, counts: np.ndarray, n_samples: int, k: int, M: float, a: float, d: float, Q: float):
    counts = np.ascontiguousarray(counts, dtype=np.uint32)
    cost = C.c_double(0.0); b = C.c_double(0.0)
    rc = lib().ora_epoch_cost(C.c_int32(T), C.c_int64(counts.shape[0]), _p(counts), C.c_int64(n_samples), C.c_int64(k),
                              C.c_double(M), C.c_double(a), C.c_double(d), C.c_double(Q), C.byref(cost), C.byref(b))
    return rc, cost.value, b.value


def caching_gain(counts: np.ndarray, n_samples: int, k: int, M: float, a: float, d: float):
    counts = np.ascontiguousarray(counts, dtype=np.uint32)
    lhs = C.c_double(0.0); t1 = C.c_double(0.0)
    rc = lib().ora_caching_gain(C.c_int64(counts.shape[0]), _p(counts), C.c_int64(n_samples), C.c_int64(k), C.c_double(M),
                                C.c_double(a), C.c_double(d), C.byref(lhs), C.byref(t1))
    return rc, lhs.value, t1.value


def plan_brute(T: int, counts: np.ndarray, n_samples: int, k_max: int, M: float, a: float, d: float, Q: float):
    counts = np.ascontiguousarray(counts, dtype=np.uint32)
    bk = C.c_int64(0); bc = C.c_double(0.0)
    rc = lib().ora_plan_brute(C.c_int32(T), C.c_int64(counts.shape[0]), _p(counts), C.c_int64(n_samples), C.c_int64(k_max),
                              C.c_double(M), C.c_double(a), C.c_double(d), C.c_double(Q), C.byref(bk), C.byref(bc))
    return rc, bk.value, bc.value


def _dt(tables: Sequence[np.ndarray]) -> Tuple[int, int]:
    d = tables[0].dtype
    assert d in (np.float32, np.uint16), "rows are fp32, or bf16 held as uint16"
    return (0 if d == np.float32 else 1), int(tables[0].shape[1])


def embedding_bag_fwd(rows, tables: Sequence[np.ndarray], indices, offsets, B: int,
                      slot_of: Optional[np.ndarray] = None, cache: Optional[np.ndarray] = None):
    rows = _rows(rows); indices = _i32(indices); offsets = _i32(offsets)
    T = _LB(rows, offsets, B)
    dtype, D = _dt(tables)
    out = np.empty((T * B, D), dtype=np.float32)
    tp = _ptr_array(tables)
    if slot_of is None:
        rc = lib().ora_embedding_bag_fwd(C.c_int32(T), _p(rows), C.c_int32(D), C.c_int32(dtype), tp, _p(indices),
                                         _p(offsets), C.c_int64(indices.shape[0]), C.c_int64(B), _p(out))
    else:
        rc = lib().ora_embedding_bag_fwd_cached(C.c_int32(T), _p(rows), C.c_int32(D), C.c_int32(dtype), tp,
                                                _p(_i32(slot_of)), _p(cache), _p(indices), _p(offsets),
                                                C.c_int64(indices.shape[0]), C.c_int64(B), _p(out))
    return rc, out


def bwd_segments(rows, indices, offsets, B: int):
    rows = _rows(rows); indices = _i32(indices); offsets = _i32(offsets)
    T = _LB(rows, offsets, B)
    L = indices.shape[0]
    sg = np.empty(L, dtype=np.int32); sb = np.empty(L, dtype=np.int32)
    ss = np.empty(L + 1, dtype=np.int32); ug = np.empty(L, dtype=np.int32)
    U = np.zeros(1, dtype=np.int64)
    rc = lib().ora_bwd_segments(C.c_int32(T), _p(rows), _p(indices), _p(offsets), C.c_int64(L), C.c_int64(B),
                                _p(sg), _p(sb), _p(ss), _p(ug), _p(U))
    if rc not in (OK, ERR_INDEX_RANGE):
        return rc, None, None, None, None
    u = int(U[0]); n = int(ss[u])
    return rc, sg[:n].copy(), sb[:n].copy(), ss[: u + 1].copy(), ug[:u].copy()


def embedding_bag_bwd_update(rows, tables: Sequence[np.ndarray], state: Optional[Sequence[np.ndarray]],
                             optimizer: int, indices, offsets, B: int, grad_out: np.ndarray, lr: float,
                             eps: float, report: bool = False, n_unique: int = 0, want_outputs: bool = True):
    """report=False mutates `tables`/`state` in place and returns (rc,).  report=True mutates nothing and
    returns (rc, new_rows, new_state, grad_rows) as fp64 [n_unique, D] arrays (n_unique from bwd_segments)."""
    rows = _rows(rows); indices = _i32(indices); offsets = _i32(offsets)
    T = _LB(rows, offsets, B)
    dtype, D = _dt(tables)
    grad_out = np.ascontiguousarray(grad_out, dtype=np.float32)
    assert grad_out.shape == (T * B, D)
    tp = _ptr_array(tables)
    sp = _ptr_array(state) if state is not None else None
    nr = ns = gr = None
    if report and want_outputs:
        nr = np.zeros((n_unique, D), dtype=np.float64)
        ns = np.zeros((n_unique, D), dtype=np.float64)
        gr = np.zeros((n_unique, D), dtype=np.float64)
    rc = lib().ora_embedding_bag_bwd_update(C.c_int32(T), _p(rows), C.c_int32(D), C.c_int32(dtype), tp, sp,
                                            C.c_int32(optimizer), _p(indices), _p(offsets),
                                            C.c_int64(indices.shape[0]), C.c_int64(B), _p(grad_out),
                                            C.c_float(lr), C.c_float(eps), C.c_int32(1 if report else 0),
                                            _p(nr), _p(ns), _p(gr))
    if report:
        return rc, nr, ns, gr
    return (rc,)
