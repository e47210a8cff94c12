"""The library's host side (argument checks, size queries, bookkeeping, the C caller) once more with the host code built
under AddressSanitizer and UndefinedBehaviorSanitizer.  Device code is compiled as usual and never runs here."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_logic_passes_with_the_host_code_under_asan_and_ubsan(tmp_path):
    sys.path.insert(0, ROOT)
    from paper_2411_01611_amd import build as hip_build
    asan = hip_build.asan_runtime()
    if not asan:
        pytest.skip("hipcc's clang has no shared AddressSanitizer runtime here")
    lib = hip_build.build(out_dir=str(tmp_path), host_sanitize=True)
    env = dict(os.environ)
    env["LD_PRELOAD"] = ":".join(x for x in (env.get("LD_PRELOAD", ""), asan) if x)   # whatever is preloaded stays, in front
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:exitcode=99"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["SCARS_LIB_PATH"] = lib
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_host_logic.py"),
                        "--deselect", "tests/test_host_logic.py::test_bench_refuses_more_than_one_gpu"],
                       env=env, cwd=ROOT, capture_output=True, text=True, timeout=900)
    tail = r.stdout[-3000:] + "\n" + r.stderr[-3000:]
    assert r.returncode == 0, tail
    assert " passed" in r.stdout and "failed" not in r.stdout, tail
    probe = subprocess.run([sys.executable, "-c", "from paper_2411_01611_amd import binding; print(binding.lib()._name)"],
                           env=env, cwd=ROOT, capture_output=True, text=True, timeout=300)
    assert probe.returncode == 0 and probe.stdout.strip() == lib, probe.stdout + probe.stderr
