"""The C ABI's host code under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU: every call in the
driver fails validation before anything is launched, or is a pure-host size query).

The boundary's translation units (argument validation, dispatch, the library-owned scratch entry point) are
recompiled with the sanitizers on their host side only and linked with the already built kernel objects."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
PKG = os.path.join(ROOT, "paper_2102_05743_amd")
SANITIZED = ["api.hip", "small_d.hip", "static_scratch.hip", "ktimer.hip", "blocks.hip"]
HIP_FLAGS = ["-O1", "-g", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
             "-packed-fp32-ops", "-Wno-unused-command-line-argument",
             "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-sanitize-recover=all"]


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not available")
def test_boundary_clean_under_asan_and_ubsan(tmp_path):
    objdir = os.path.join(PKG, "_build")
    if not os.path.isdir(objdir):
        pytest.skip("the library's objects are not built (python -m paper_2102_05743_amd.build)")
    objs = []
    for src in SANITIZED:
        obj = str(tmp_path / (src + ".o"))
        r = subprocess.run(["hipcc", *HIP_FLAGS, "-c", os.path.join(PKG, "csrc", src), "-o", obj],
                           capture_output=True, text=True)
        assert r.returncode == 0, r.stderr
        objs.append(obj)
    from paper_2102_05743_amd import build
    taken = {s.replace(".hip", ".o") for s in SANITIZED}
    objs += [os.path.join(objdir, name) for _, _, name in build.UNITS if name not in taken]   # the main library's units
    lib = str(tmp_path / "libhmmscan_san.so")
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address,undefined",
                        "-fno-gpu-sanitize", "-o", lib, *objs], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    exe = str(tmp_path / "sanitize_boundary")
    clang = "/opt/rocm/llvm/bin/clang" if os.path.exists("/opt/rocm/llvm/bin/clang") else "amdclang"
    r = subprocess.run([clang, "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                        os.path.join(HERE, "sanitize_boundary_driver.c"), lib, "-Wl,-rpath," + str(tmp_path), "-o", exe],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:protect_shadow_gap=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "ok" in run.stdout
