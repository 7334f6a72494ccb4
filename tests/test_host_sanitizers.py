"""The library's host side (argument validation, plan selection, selective-precision bookkeeping: integer divisions and
shape-derived loops) under AddressSanitizer and UndefinedBehaviorSanitizer on the CPU.  The C-ABI translation unit is
rebuilt with the sanitizers on the host pass only (GPU AddressSanitizer is not used), linked with the kernels' ordinary
objects into a small driver (tests/host/plan_sanitize_driver.cpp) that calls only entry points which launch nothing."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2505_15909_amd")


def test_planning_and_validation_are_clean_under_asan_and_ubsan(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    objs = [os.path.join(PKG, "_build", f) for f in ("rtn_quantize.o", "rtn_linear.o", "rtn_linear_wide.o", "rtn_gemm_tile.o", "rtn_bench.o")]
    if not all(os.path.exists(o) for o in objs):
        pytest.skip("library objects not built (run __graft_entry__.build() first)")
    # sanitizers on the host pass only: every -fsanitize= option directly follows -Xarch_host
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined",
           "-Xarch_host", "-fno-omit-frame-pointer"]
    common = ["-O1", "-g", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
    api_o = str(tmp_path / "rtn_api_san.o")
    drv_o = str(tmp_path / "driver_san.o")
    exe = str(tmp_path / "plan_sanitize_driver")
    subprocess.run([hipcc, *common, *san, "-c", "-o", api_o, os.path.join(PKG, "csrc", "rtn_api.hip")], check=True, cwd=os.path.join(PKG, "csrc"),
                   capture_output=True, timeout=600)
    subprocess.run([hipcc, *common, *san, "-x", "hip", "-c", "-o", drv_o, os.path.join(ROOT, "tests", "host", "plan_sanitize_driver.cpp")],
                   check=True, capture_output=True, timeout=600)
    subprocess.run([hipcc, "--offload-arch=gfx950", *san, "-o", exe, drv_o, api_o, *objs], check=True, capture_output=True, timeout=600)
    env = dict(os.environ)
    # leaks are not what is tested here (the HIP runtime keeps its own allocations until exit); everything else aborts;
    # a library preloaded ahead of the sanitizer runtime is tolerated
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:halt_on_error=1:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    r = subprocess.run([exe], capture_output=True, text=True, timeout=900, env=env)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]
    assert "automatic plans validated" in r.stdout
