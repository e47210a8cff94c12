"""The oracle's pins once more, with the oracle built under AddressSanitizer and UndefinedBehaviorSanitizer: an
out-of-bounds access, a use after free, a signed overflow or a misaligned access in scars_oracle.c ends the run."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_pins_pass_under_asan_and_ubsan(tmp_path):
    if not shutil.which("gcc"):
        pytest.skip("no gcc")
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("gcc has no libasan here")
    so = str(tmp_path / "liboracle_san.so")
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
                           "-o", so, os.path.join(ROOT, "oracle", "scars_oracle.c"), "-lm"])
    env = dict(os.environ)
    # the sanitizer runtime has to be in the process before the instrumented library is loaded; whatever is
    # preloaded already stays, in front
    env["LD_PRELOAD"] = ":".join(x for x in (env.get("LD_PRELOAD", ""), asan) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0:exitcode=99"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["SCARS_ORACLE_SO"] = so
    env["OMP_NUM_THREADS"] = "4"
    tests = [os.path.join(ROOT, "tests", f) for f in ("test_oracle_golden.py", "test_oracle_integer.py",
                                                       "test_oracle_float.py", "test_oracle_cost_model.py")]
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *tests], env=env, cwd=ROOT,
                       capture_output=True, text=True, timeout=900)
    tail = (r.stdout[-3000:] + "\n" + r.stderr[-3000:])
    assert r.returncode == 0, tail
    assert " passed" in r.stdout and "failed" not in r.stdout, tail
    # the instrumented library is really the one that ran
    probe = subprocess.run([sys.executable, "-c", "import oracle, ctypes; l = oracle.lib(); print(l._name)"], env=env, cwd=ROOT,
                           capture_output=True, text=True, timeout=300)
    assert probe.returncode == 0 and probe.stdout.strip() == so, probe.stdout + probe.stderr
