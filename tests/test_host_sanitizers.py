"""The boundary's host logic under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

The library's sources are compiled once more with sanitizers on the HOST side only (the device code is built but never run),
linked with tests/host_sanitize/driver.cpp, and that program exercises what the host does before any launch: descriptor
checks, ring arithmetic against a brute-force ring, size functions, the argument checks of every entry point."""
import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2512_04677_amd", "csrc")
HIPCC = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
SOURCES = ["lvx_cache", "lvx_rope_norm", "lvx_attention", "lvx_gemm", "lvx_fp8", "lvx_conv", "lvx_block"]
HOST_SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not found")
def test_host_logic_is_clean_under_asan_and_ubsan(tmp_path):
    common = [HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
              "-packed-fp32-ops", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]

    def compile_one(name):
        out = str(tmp_path / (name + ".o"))
        r = subprocess.run(common + HOST_SAN + ["-c", os.path.join(CSRC, name + ".hip"), "-o", out], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        return out

    with ThreadPoolExecutor(max_workers=4) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    drv = str(tmp_path / "driver.o")
    r = subprocess.run(common + HOST_SAN + ["-x", "hip", os.path.join(ROOT, "tests", "host_sanitize", "driver.cpp"), "-c", "-o", drv],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    exe = str(tmp_path / "driver")
    r = subprocess.run([HIPCC, "--offload-arch=gfx950"] + HOST_SAN + ["-o", exe, drv] + objs, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    env = dict(os.environ)
    # leaks: the HIP runtime's own start-up allocations; link order: other preloaded libraries may come before the runtime
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1"
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert "host checks passed" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]
