"""Builds the C-ABI shared library (HIP kernels for gfx950 + host runtime) in-tree."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_NAME = "libautochunk_rt.so"
LIB_PATH = os.path.join(HERE, LIB_NAME)

SOURCES = ["rowwise.hip", "linear.hip", "attention.hip", "runtime.hip", "search.hip"]

# Per-file extras.  attention.hip: keep MFMA results in VGPRs; the softmax reads every score
# right after the matrix op, and accumulator-register copies would double its VALU work.
# search.hip (host only): its cost function is compared bit for bit, so no fused multiply-adds.
EXTRA_FLAGS = {"attention.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"], "search.hip": ["-ffp-contract=off"]}

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def _hipcc() -> str:
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cand = os.path.join(rocm, "bin", "hipcc")
    return cand if os.path.exists(cand) else "hipcc"


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), r.stdout))
    return r.stdout


def build(verbose: bool = False, jobs: int = 4) -> str:
    """Compile every source for gfx950 and link the shared library; returns its path."""
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    hipcc = _hipcc()

    def compile_one(src):
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        out = _run([hipcc, *HIPCC_FLAGS, *EXTRA_FLAGS.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj])
        if verbose and out.strip():
            print(out)
        return obj

    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH, *objs])
    return LIB_PATH


def ensure_built() -> str:
    """The library's path, compiling it first only if no built library is there (for the test
    suite, the smoke run and the benchmark; the binding itself never builds and raises)."""
    return LIB_PATH if os.path.exists(LIB_PATH) else build()


if __name__ == "__main__":
    print(build(verbose=True))
