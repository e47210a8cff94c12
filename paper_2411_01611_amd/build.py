"""Build libscars.so (HIP, gfx950) in-tree with hipcc.  `python -m paper_2411_01611_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libscars.so")
SOURCES = ["scars_api.hip", "k_sort.hip", "k_build_cache.hip", "k_remap.hip", "k_classify.hip", "k_plan.hip", "k_fwd.hip", "k_bwd.hip"]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    raise RuntimeError("hipcc not found")


# host code only (GPU-side sanitizers are not used): AddressSanitizer and UndefinedBehaviorSanitizer for the
# library's argument checks, bookkeeping and planning arithmetic
HOST_SANITIZE = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
                 "-fno-omit-frame-pointer", "-g"]


def build(verbose: bool = False, out_dir: str = None, host_sanitize: bool = False) -> str:
    """Compile every source and link libscars.so: in-tree by default, or into out_dir (objects beside the library)."""
    obj_dir = os.path.join(out_dir, "_build") if out_dir else OBJ
    lib = os.path.join(out_dir, "libscars.so") if out_dir else LIB
    os.makedirs(obj_dir, exist_ok=True)
    cc = _hipcc()
    flags = [f for f in FLAGS if f != "-O3"] + ["-O1"] + HOST_SANITIZE if host_sanitize else FLAGS

    def one(src: str) -> str:
        obj = os.path.join(obj_dir, src.replace(".hip", ".o"))
        cmd = [cc, *flags, "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0 or verbose:
            sys.stderr.write(r.stdout + r.stderr)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}")
        return obj

    with ThreadPoolExecutor(max_workers=min(6, os.cpu_count() or 1)) as ex:
        objs = list(ex.map(one, SOURCES))
    link = ["-fsanitize=address", "-shared-libsan"] if host_sanitize else []
    subprocess.check_call([cc, "--offload-arch=gfx950", "-shared", "-fPIC", *link, "-o", lib, *objs])
    return lib


def asan_runtime() -> str:
    """The shared AddressSanitizer runtime of hipcc's clang (to be preloaded into a process that loads a
    host-sanitized build), or '' if it cannot be found."""
    r = subprocess.run([_hipcc(), "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True)
    p = r.stdout.strip()
    return p if os.path.isabs(p) and os.path.exists(p) else ""


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
