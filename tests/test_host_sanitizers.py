"""The host side of liblsw under AddressSanitizer + UndefinedBehaviorSanitizer: lsw_api.cpp is compiled with both (host code
only; the device code of the already built library is linked as it is) together with tests/host_sanitizer_driver.cpp, which
drives every entry point that can run without a device.  Any report aborts the driver (-fno-sanitize-recover)."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2405_17741_amd")


def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc) or not os.path.exists(os.path.join(PKG, "liblsw.so")):
        pytest.skip("needs hipcc and the built library")
    exe = str(tmp_path / "host_sanitizer_driver")
    cmd = [hipcc, "-O1", "-g", "-std=c++17", "--offload-arch=gfx950",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG, "csrc"),
           "-x", "hip", os.path.join(ROOT, "tests", "host_sanitizer_driver.cpp"), os.path.join(PKG, "csrc", "lsw_api.cpp"),
           "-x", "none", "-L", PKG, "-l:liblsw.so", "-Wl,-rpath," + PKG, "-o", exe]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-3000:]
    env = dict(os.environ)
    # another library may be preloaded ahead of the sanitizer runtime; leaks of the HIP runtime itself are not ours
    env["ASAN_OPTIONS"] = "verify_asan_link_order=0:detect_leaks=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1"
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-3000:])
    assert "host sanitizer driver OK" in run.stdout
