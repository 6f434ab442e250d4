"""Sanitizer builds (address + undefined behaviour, host code only) of the C controller and of the argument checks of
the C ABI: compiled here, run on the CPU; no call reaches the GPU."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
INC = os.path.join(ROOT, "include")
CSRC = os.path.join(ROOT, "paper_2504_00030_amd", "csrc")
DRIVER = os.path.join(ROOT, "tests", "sanitize", "driver.c")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def _run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert r.returncode == 0, " ".join(cmd) + "\n" + r.stdout[-4000:]
    return r.stdout


def test_controller_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "gt_san")
    _run(["gcc", "-std=gnu11", "-O1", "-g", "-ffp-contract=off", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
          "-I" + INC, DRIVER, os.path.join(CSRC, "gammatune.c"), "-lm", "-o", exe])
    out = _run([exe, "controller", os.path.join(ROOT, "tests", "golden", "gammatune_trajectories.txt")], env=ENV)
    assert "FAILED" not in out and "runtime error" not in out and "AddressSanitizer" not in out


def test_api_argument_checks_under_address_and_ub_sanitizers(tmp_path):
    """engine.hip's host code compiled with the sanitizers and linked with the kernels' ordinary objects (as built by
    paper_2504_00030_amd.build); every call of the driver must be refused on its arguments."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    build = os.path.join(ROOT, "paper_2504_00030_amd", "_build")
    objs = [os.path.join(build, f) for f in sorted(os.listdir(build))] if os.path.isdir(build) else []
    objs = [o for o in objs if o.endswith(".o") and "engine" not in os.path.basename(o)]
    if not shutil.which(hipcc) or len(objs) < 6:
        pytest.skip("needs hipcc and the library's objects (python -m paper_2504_00030_amd.build)")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all"]
    eng = str(tmp_path / "engine_san.o")
    _run([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-fno-gpu-rdc", "-Xclang", "-target-feature",
          "-Xclang", "-packed-fp32-ops", *san, "-I" + INC, "-I" + CSRC, "-c", os.path.join(CSRC, "engine.hip"), "-o", eng])
    drv = str(tmp_path / "driver.o")
    _run(["gcc", "-std=gnu11", "-O1", "-g", "-DWITH_API", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-I" + INC,
          "-c", DRIVER, "-o", drv])
    exe = str(tmp_path / "api_san")
    _run([hipcc, "--offload-arch=gfx950", *san, eng, drv, *objs, "-o", exe])
    out = _run([exe, "api"], env=ENV)
    assert "FAILED" not in out and "runtime error" not in out and "AddressSanitizer" not in out
