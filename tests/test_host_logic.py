"""CPU-side checks of the C ABI: the library loads, exports every declared symbol, and its host-only logic
(configuration checks, size queries, call-order errors) behaves.  No kernel is launched."""
import ctypes as C
import os
import re

import pytest

from paper_2411_01611_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "scars.h")).read()
    declared = set(re.findall(r"\b(scars_[a-z_]+)\s*\(", header))
    declared -= {"scars_handle"}
    assert declared == set(binding.EXPORTS)
    L = binding.lib()
    for name in declared:
        assert hasattr(L, name), name


def _cfg(rows, dim, dtype=0, opt=0, tables=None, state=None):
    T = len(rows)
    rows_a = (C.c_int64 * T)(*rows)
    tabs = (C.c_void_p * T)(*(tables or [0x1000] * T))
    st = (C.c_void_p * T)(*state) if state else None
    return binding._Config(T, rows_a, dim, dtype, tabs, opt, st), (rows_a, tabs, st)


def test_create_rejects_bad_configurations():
    L = binding.lib()
    h = C.c_void_p()
    for rows, dim, dtype, opt, tables, state in (
        ([], 16, 0, 0, None, None),                 # no tables
        ([10], 3, 0, 0, None, None),                # row bytes not a multiple of 16
        ([10], 4, 1, 0, None, None),                # bf16 dim 4 = 8 bytes
        ([10], 512, 0, 0, None, None),              # row larger than 1024 bytes
        ([10], 16, 2, 0, None, None),               # unknown dtype
        ([10], 16, 0, 3, None, None),               # unknown optimizer
        ([10], 16, 0, 1, None, None),               # Adagrad without state
        ([10, 0], 16, 0, 0, None, None),            # empty table
        ([2 ** 30, 2 ** 30], 16, 0, 0, None, None),  # 2^31 rows
        ([10], 16, 0, 0, [0], None),                # null table pointer
    ):
        cfg, keep = _cfg(rows, dim, dtype, opt, tables, state)
        assert L.scars_create(C.byref(cfg), C.byref(h)) == binding.ERR_INVALID_ARG
    assert L.scars_create(None, C.byref(h)) == binding.ERR_INVALID_ARG


def test_query_sizes_and_budget_rows():
    s = binding.Scars([1000, 3000], 64, binding.DTYPE_F32, [0x1000, 0x2000])
    z = s.query_sizes(0, 100, 10)
    assert z["k"] == 0
    assert s.query_sizes(255, 100, 10)["k"] == 0                   # budget below one row
    assert s.query_sizes(256, 100, 10)["k"] == 1
    assert s.query_sizes(256 * 4000 + 17, 100, 10)["k"] == 4000
    assert s.query_sizes(10 ** 12, 100, 10)["k"] == 4000
    z = s.query_sizes(256 * 500, 5000, 2000)
    assert z["counts_bytes"] >= 4000 * 4 and z["slot_of_bytes"] >= 4000 * 4
    assert z["cache_bytes"] >= 500 * 256 and z["state_cache_bytes"] == 0
    assert z["workspace_bytes"] >= 5000 * 256                      # staging for max_L rows
    assert z["out_bytes"] >= 2000 * 64 * 4 and z["seg_start_bytes"] >= 5001 * 4
    assert all(v % 256 == 0 for k, v in z.items() if k.endswith("_bytes"))
    with pytest.raises(binding.ScarsError):
        s.query_sizes(-1, 1, 1)
    with pytest.raises(binding.ScarsError):
        s.query_sizes(0, 2 ** 31, 1)
    sa = binding.Scars([1000], 64, binding.DTYPE_F32, [0x1000], binding.OPT_ADAGRAD, [0x3000])
    assert sa.query_sizes(256 * 10, 1, 1)["state_cache_bytes"] >= 10 * 256
    sb = binding.Scars([1000], 64, binding.DTYPE_BF16, [0x1000])
    assert sb.query_sizes(128 * 10, 1, 1)["k"] == 10


def test_calls_before_bind_report_workspace_error():
    L = binding.lib()
    s = binding.Scars([100], 16, binding.DTYPE_F32, [0x1000])
    assert L.scars_build_cache(s._h, None, None, 0, 0, 0, 0, None) == binding.ERR_WORKSPACE
    assert L.scars_remap(s._h, None, None, 0, 0, None, None) == binding.ERR_WORKSPACE
    assert L.scars_flush_cache(s._h, None) == binding.ERR_WORKSPACE
    assert L.scars_sync_status(s._h, None) == binding.ERR_WORKSPACE
    assert b"no buffers bound" in L.scars_last_error(s._h)
    assert L.scars_cache_rows(s._h) == -1
    assert L.scars_remap(None, None, None, 0, 0, None, None) == binding.ERR_INVALID_ARG
    assert L.scars_destroy(None) == binding.ERR_INVALID_ARG


def test_tuning_counters_and_planning_calls_check_their_arguments():
    L = binding.lib()
    s = binding.Scars([100], 16, binding.DTYPE_F32, [0x1000])
    s.set_tuning(binding.TUNE_FUSED_SCAN_MAX_TILES, 0)
    s.set_tuning(binding.TUNE_FUSED_SCAN_MAX_TILES, 10 ** 6)          # clamped to the documented maximum
    s.set_tuning(binding.TUNE_PRESORT, 131072)
    s.set_tuning(binding.TUNE_PRESORT, 0)
    s.set_tuning(binding.TUNE_FUSED_LONG_MAX_L, 0)
    s.set_tuning(binding.TUNE_FUSED_LONG_MAX_L, 262144)
    s.set_tuning(binding.TUNE_PAIRS_IN_REMAP, 0)
    s.set_tuning(binding.TUNE_PAIRS_IN_REMAP, 1)
    s.set_tuning(binding.TUNE_UPDATE_MAX_BLOCKS, 256)
    for which, value in ((99, 1), (binding.TUNE_PRESORT, -1), (binding.TUNE_PRESORT, 2 ** 31)):
        assert L.scars_set_tuning(s._h, which, value) == binding.ERR_INVALID_ARG
    assert L.scars_set_tuning(None, binding.TUNE_PRESORT, 1) == binding.ERR_INVALID_ARG
    assert s.get_counter(binding.COUNTER_PREPARED_USED) == 0
    assert L.scars_get_counter(s._h, 99) == -1 and L.scars_get_counter(None, 1) == -1
    # planning before any buffer is bound
    pin = binding._PlanIn(1e6, 1e3, 1e5, 100)
    po = binding._PlanOut()
    cost, b = C.c_double(0.0), C.c_double(0.0)
    assert L.scars_plan_cache(s._h, C.byref(pin), C.byref(po), None) == binding.ERR_WORKSPACE
    assert L.scars_epoch_cost(s._h, C.byref(pin), 0, C.byref(cost), C.byref(b), None) == binding.ERR_WORKSPACE
    assert L.scars_plan_cache(None, C.byref(pin), C.byref(po), None) == binding.ERR_INVALID_ARG


def test_bind_buffers_refuses_buffers_smaller_than_query_sizes_asks_for():
    """Every buffer handed to scars_bind_buffers carries its size; one byte short of what scars_query_sizes asks for
    with the same three arguments is refused before anything touches the device."""
    L = binding.lib()
    for opt, state in ((binding.OPT_SGD, None), (binding.OPT_ADAGRAD, [0x3000, 0x4000])):
        s = binding.Scars([1000, 3000], 64, binding.DTYPE_F32, [0x1000, 0x2000], opt, state)
        budget, max_L, max_G = 256 * 500, 4096, 512
        z = s.query_sizes(budget, max_L, max_G)
        names = ["counts", "slot_of", "hot_gid", "cache", "state_cache", "workspace"]
        full = [z[n + "_bytes"] for n in names]
        ptr = lambda n: None if (n == "state_cache" and opt == binding.OPT_SGD) else 0x10000
        for short in names:
            if short == "state_cache" and opt == binding.OPT_SGD:
                continue
            sizes = [v - 1 if n == short else v for n, v in zip(names, full)]
            b = binding._Buffers(*[ptr(n) for n in names], budget, max_L, max_G, *sizes)
            assert L.scars_bind_buffers(s._h, C.byref(b), None) == binding.ERR_WORKSPACE, short
            assert b"smaller" in L.scars_last_error(s._h)
        # binding a larger budget or batch than the buffers were sized for is the same mistake
        for bud, ml, mg in ((budget * 2, max_L, max_G), (budget, max_L * 2, max_G), (budget, max_L, max_G * 4096)):
            b = binding._Buffers(*[ptr(n) for n in names], bud, ml, mg, *full)
            assert L.scars_bind_buffers(s._h, C.byref(b), None) == binding.ERR_WORKSPACE
        s.close()


def test_bench_refuses_more_than_one_gpu():
    """bench.py --gpus N with N > 1 (or a multi-rank launch) exits with a message instead of running."""
    import subprocess
    import sys
    for argv, env in ((["--gpus", "2"], {}), ([], {"WORLD_SIZE": "2"})):
        r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *argv], capture_output=True, text=True,
                           env={**os.environ, **env}, timeout=300)
        assert r.returncode == 2
        assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


C_PROGRAM = r"""
#include <stdio.h>
#include "scars.h"

int main(void) {
    int64_t rows[2] = {1000, 50};
    static char t0[16], t1[16];
    void* tables[2] = {t0, t1};
    scars_config cfg;
    scars_handle* h = NULL;
    scars_sizes sz;
    cfg.num_tables = 2; cfg.rows = rows; cfg.dim = 32; cfg.dtype = SCARS_DTYPE_F32;
    cfg.host_tables = tables; cfg.optimizer = SCARS_OPT_SGD; cfg.host_state = NULL;
    if (scars_create(&cfg, &h) != SCARS_OK) return 1;
    if (scars_query_sizes(h, 100 * 128, 4096, 512, &sz) != SCARS_OK) return 2;
    printf("%lld %lld %lld\n", (long long)sz.k, (long long)sz.cache_bytes, (long long)sz.out_bytes);
    if (scars_cache_rows(h) != -1) return 3;
    cfg.dim = 3;                                    /* 12-byte rows: refused */
    { scars_handle* bad = NULL; if (scars_create(&cfg, &bad) != SCARS_ERR_INVALID_ARG || bad) return 4; }
    return scars_destroy(h) == SCARS_OK ? 0 : 5;
}
"""


def test_header_is_plain_c_and_a_c_program_links_against_the_library(tmp_path):
    """include/scars.h compiles as strict C99 with no other include, and a C caller with no Python or torch in the
    process can create a handle, query sizes and destroy it."""
    import shutil
    import subprocess
    if not shutil.which("gcc"):
        pytest.skip("no gcc")
    src = tmp_path / "caller.c"
    src.write_text(C_PROGRAM)
    exe = tmp_path / "caller"
    libdir = os.path.dirname(binding.LIB_PATH)
    subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"),
                           str(src), "-o", str(exe), "-L", libdir, "-lscars", "-Wl,-rpath," + libdir,
                           "-Wl,--allow-shlib-undefined"])
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stderr
    k, cache_bytes, out_bytes = (int(x) for x in r.stdout.split())
    assert k == 100 and cache_bytes >= 100 * 128 and out_bytes >= 512 * 32 * 4


def test_update_kernels_keep_their_registers(tmp_path):
    """The update kernels share a launch between several jobs (rows, long runs, the fetch of the next batch): the
    widest job sets the registers of all of them.  The compiler's own figures for every instantiation: no spills,
    and the instantiations that large batches run keep at least five waves per SIMD (a fully unrolled reduction in
    one job once took that to three, and the bandwidth-bound part of the launch with it)."""
    import re
    import subprocess
    from paper_2411_01611_amd import build
    src = os.path.join(build.CSRC, "k_bwd.hip")
    cmd = [build._hipcc(), *build.FLAGS, "--cuda-device-only", "-c", src, "-o", str(tmp_path / "k_bwd.o"),
           "-Rpass-analysis=kernel-resource-usage"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    seen = 0
    for block in re.split(r"remark: Function Name: ", r.stderr)[1:]:
        name = block.split()[0]
        num = lambda key: int(re.search(key + r": (\d+)", block).group(1))
        vgprs, waves, scratch = num("VGPRs"), num(r"Occupancy \[waves/SIMD\]"), num(r"ScratchSize \[bytes/lane\]")
        assert scratch == 0, (name, scratch)
        m = re.search(r"k_seg_rows_longILi\dELi\dELi\d+ELi(\d+)ELb", name)
        if m:
            seen += 1
            # (4: the instantiation of batches above 131072 lookups; 16: small batches, wide long-run part)
            assert waves >= (5 if m.group(1) == "4" else 3), (name, vgprs, waves)
        elif "14k_small_update" in name or "10k_seg_rowsI" in name:
            seen += 1
            assert waves >= 5, (name, vgprs, waves)
    assert seen >= 3 * 32, seen
