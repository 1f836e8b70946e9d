"""Build libe0m4.so (HIP, gfx950) in-tree with hipcc.  No GPU is needed to build."""
from __future__ import annotations

import concurrent.futures
import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(ROOT, "include")
BUILD_DIR = os.path.join(HERE, "_build")
LIB_PATH = os.path.join(HERE, "libe0m4.so")

SOURCES = ["e0m4_api.hip", "e0m4_pack.hip", "e0m4_gemv.hip", "e0m4_gemv_mfma.hip", "e0m4_gemv_dq.hip", "e0m4_gemm.hip", "e0m4_gemm_pipe.hip",
           "e0m4_norm.hip", "e0m4_kv.hip", "e0m8_pack.hip"]
# the quantiser's fp32 steps must stay single IEEE operations
EXTRA_FLAGS = {"e0m4_pack.hip": ["-ffp-contract=off"], "e0m8_pack.hip": ["-ffp-contract=off"]}

COMMON_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
    "-I", INCLUDE, "-I", CSRC,
    # packed fp32 instructions are kept out of all device code on this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the first kernel arguments (14 scalar registers' worth) arrive in registers with the launch instead of
    # through a load at the start of every wavefront: 0.2 - 0.4 us per launch of the decode kernels
    "-mllvm", "-amdgpu-kernarg-preload-count=16",
    "-Wno-unused-command-line-argument",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def _compile(src: str, extra=()) -> str:
    obj = os.path.join(BUILD_DIR, src.replace(".hip", ".o"))
    cmd = [hipcc(), *COMMON_FLAGS, *EXTRA_FLAGS.get(src, []), *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, r.stdout, r.stderr))
    lines = [l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip()]
    if lines:
        print("\n".join(lines))
    return obj


def build_library(extra_flags=(), verbose: bool = True) -> str:
    os.makedirs(BUILD_DIR, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(lambda s: _compile(s, extra_flags), SOURCES))
    tmp = LIB_PATH + ".tmp.%d" % os.getpid()
    subprocess.check_call([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", tmp])
    os.replace(tmp, LIB_PATH)
    if verbose:
        print("built", LIB_PATH)
    return LIB_PATH


if __name__ == "__main__":
    build_library()
