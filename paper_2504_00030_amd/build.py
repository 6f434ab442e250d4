"""Build libspecdecode.so (HIP kernels + host engine + C controller) for gfx950, in-tree.

    python -m paper_2504_00030_amd.build

hipcc cross-compiles without a GPU.  Objects go to paper_2504_00030_amd/_build/,
the library to paper_2504_00030_amd/lib/libspecdecode.so.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

if __package__:
    from . import isa_guard
else:  # run as a script
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    import isa_guard

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
BUILD = os.path.join(PKG, "_build")
LIBDIR = os.path.join(PKG, "lib")
LIB = os.path.join(LIBDIR, "libspecdecode.so")

HIP_SOURCES = [
    "engine.hip",
    "kernels/gemv_wavedot.hip",
    "kernels/gemv_mfma.hip",
    "kernels/gemm_mfma.hip",
    "kernels/attention.hip",
    "kernels/sampler.hip",
    "kernels/misc.hip",
]
C_SOURCES = ["gammatune.c"]
MFMA_SOURCES = ["kernels/gemv_mfma.hip", "kernels/gemm_mfma.hip", "kernels/attention.hip"]  # scanned by isa_guard after compiling

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
HIP_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-Wall", "-Wno-unused-function",
]
C_FLAGS = ["-O2", "-fPIC", "-ffp-contract=off", "-std=c11", "-Wall", "-I" + os.path.join(ROOT, "include")]


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("command failed: " + " ".join(cmd) + "\n" + r.stdout)
    return r.stdout


def _obj(src):
    return os.path.join(BUILD, src.replace("/", "_") + ".o")


def build(verbose: bool = True, jobs: int = 8) -> str:
    os.makedirs(BUILD, exist_ok=True)
    os.makedirs(LIBDIR, exist_ok=True)
    hip_sources = [s for s in HIP_SOURCES if os.path.exists(os.path.join(CSRC, s))]

    def compile_hip(src):
        out = _run([HIPCC, *HIP_FLAGS, "-c", os.path.join(CSRC, src), "-o", _obj(src)])
        return src, out

    def guard_hip(src):
        # second, assembly-only compile of the matrix-core kernels, scanned by isa_guard
        asm = _obj(src)[:-2] + ".s"
        _run([HIPCC, *HIP_FLAGS, "--cuda-device-only", "-S", os.path.join(CSRC, src), "-o", asm])
        with open(asm) as f:
            bad = isa_guard.scan(f.read())
        if bad:
            raise RuntimeError(f"{src}: " + "\n".join(bad[:10]))
        return src + " (matrix-instruction guard)", ""

    def compile_c(src):
        out = _run(["gcc", *C_FLAGS, "-c", os.path.join(CSRC, src), "-o", _obj(src)])
        return src, out

    with ThreadPoolExecutor(max_workers=jobs) as ex:
        futs = [ex.submit(compile_hip, s) for s in hip_sources] + [ex.submit(compile_c, s) for s in C_SOURCES]
        futs += [ex.submit(guard_hip, s) for s in hip_sources if s in MFMA_SOURCES]
        for f in futs:
            src, out = f.result()
            if verbose:
                warn = [l for l in out.splitlines() if "warning" in l and "packed-fp32-ops" not in l]
                print(f"[build] {src}" + (f"  ({len(warn)} warnings)" if warn else ""), flush=True)
    objs = [_obj(s) for s in hip_sources + C_SOURCES]
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    if verbose:
        print(f"[build] linked {LIB}", flush=True)
    return LIB


if __name__ == "__main__":
    try:
        build()
    except RuntimeError as e:
        print(e, file=sys.stderr)
        sys.exit(1)
