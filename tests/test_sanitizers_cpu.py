"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the CPU-side code (no GPU is touched): the C oracle,
and the host-only part of the C ABI (slicing rules, argument validation, workspace sizing), each driven by a
small program under tests/sanitize/.  Device code is compiled without sanitizers (host-side options only)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def run(cmd, **kw):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    out = "\n".join(l for l in res.stdout.splitlines() if "not a recognized feature" not in l)
    assert res.returncode == 0, out[-4000:]
    return out


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not installed")
def test_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    run(["gcc", "-O1", "-g", "-fopenmp", "-std=c99", "-Wall", "-Wextra", "-fsanitize=address,undefined",
         "-fno-omit-frame-pointer", "-o", exe, os.path.join(SAN, "oracle_driver.c"),
         os.path.join(ROOT, "oracle", "mlpmoe_oracle.c"), "-lm"])
    assert run([exe], env=ENV).strip().endswith("ok")


@pytest.mark.skipif(not os.path.exists("/opt/rocm/bin/hipcc"), reason="hipcc not installed")
def test_host_api_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "host_san")
    csrc = os.path.join(ROOT, "paper_2511_21089_amd", "csrc")
    srcs = [os.path.join(csrc, f) for f in ("mlpmoe_api.cpp", "kernels_generic.hip", "kernels_mfma.hip",
                                            "kernels_decode.hip", "kernels_fade.hip")]
    run(["/opt/rocm/bin/hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer",
         "-I", os.path.join(ROOT, "include"), "-I", csrc, "-x", "hip"] + srcs +
        [os.path.join(SAN, "host_api_driver.cpp"), "-o", exe])
    assert run([exe], env=ENV).strip().endswith("ok")
