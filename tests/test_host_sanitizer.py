"""Host code of the C ABI (argument checks, workspace carve-up) under AddressSanitizer and
UndefinedBehaviorSanitizer, on the CPU: csrc/api.hip is recompiled with the sanitizers applied to its host
pass only and linked with the library's other objects into a small driver that calls every entry point's
error paths and the workspace queries.  No GPU is needed: every call returns before a launch."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2403_02352_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
OTHERS = ["gemm_mfma", "gemm_simt", "attention", "qr", "stream", "alt", "ritz"]


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not available")
def test_host_paths_under_address_and_ub_sanitizers(tmp_path):
    objs = [os.path.join(CSRC, o + ".o") for o in OTHERS]
    missing = [o for o in objs if not os.path.exists(o)]
    if missing:   # the library has not been built in this tree yet: build it (also produces the objects)
        import importlib.util
        spec = importlib.util.spec_from_file_location("_atp_build", os.path.join(ROOT, "paper_2403_02352_amd", "build.py"))
        mod = importlib.util.module_from_spec(spec)
        spec.loader.exec_module(mod)
        mod.build_library(verbose=False)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all",
           "-Xarch_host", "-fno-omit-frame-pointer"]
    flags = ["--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wno-unused-command-line-argument"]
    api_o = str(tmp_path / "api_san.o")
    drv_o = str(tmp_path / "driver.o")
    exe = str(tmp_path / "host_checks")
    r = subprocess.run([HIPCC, *flags, *san, "-c", os.path.join(CSRC, "api.hip"), "-o", api_o], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    r = subprocess.run([HIPCC, "-O1", "-g", "-std=c++17", "-x", "c++", "-fno-gpu-sanitize", "-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all", "-c", os.path.join(ROOT, "tests", "host_sanitizer_driver.cpp"), "-o", drv_o],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-fno-gpu-sanitize", "-fsanitize=address", "-fsanitize=undefined", "-o", exe, drv_o, api_o, *objs],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, (r.stdout[-3000:], r.stderr[-3000:])
    assert "host checks ok" in r.stdout
