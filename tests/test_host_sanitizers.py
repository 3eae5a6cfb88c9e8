"""The C ABI's host code under AddressSanitizer and UndefinedBehaviorSanitizer.

Every source of the library is compiled for the host only, with both sanitizers, and linked with
tests/host_sanitize_driver.cpp.  No device code exists in that build (each translation unit's
device image is replaced by an empty offload bundle), so no kernel can run anywhere: a call that
passes its checks fails at the launch.  What runs is what has to be right on the host: argument
validation, size arithmetic at extreme shapes, the division of blocks among the items of a
batch and the argument tables of the launchers.  No GPU is needed.
"""
import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2412_01034_amd", "csrc")
HIPCC = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
# host code only: every sanitizer flag is bound to the host pass, and the device pass (absent here) is told to stay plain
SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
       "-fno-sanitize-recover=undefined", "-fno-gpu-sanitize"]


def _run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert r.returncode == 0, " ".join(cmd) + "\n" + r.stdout[-4000:]
    return r.stdout


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not found")
def test_c_abi_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    sources = sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))
    assert "api.hip" in sources
    common = [HIPCC, "-O1", "-g", "-std=c++17", "--offload-host-only", "-Wno-unused-command-line-argument",
              "-I", os.path.join(ROOT, "include"), "-I", CSRC] + SAN

    def compile_one(src):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        _run(common + ["-c", src, "-o", obj])
        return obj

    jobs = [os.path.join(CSRC, f) for f in sources] + [os.path.join(ROOT, "tests", "host_sanitize_driver.cpp")]
    with ThreadPoolExecutor(max_workers=8) as pool:
        objs = list(pool.map(compile_one, jobs))

    # the host objects refer to their device images by name: give each an empty offload bundle
    undefined = _run(["nm", "-u"] + objs)
    images = sorted({w for line in undefined.splitlines() for w in line.split() if w.startswith("__hip_fatbin_")})
    assert images
    stub_c = tmp_path / "empty_device_images.c"
    stub_c.write_text("".join(
        '__attribute__((aligned(4096))) const char %s[32] = "__CLANG_OFFLOAD_BUNDLE__";\n' % s for s in images))
    stub_o = str(tmp_path / "empty_device_images.o")
    _run(["gcc", "-c", str(stub_c), "-o", stub_o])

    exe = str(tmp_path / "host_sanitize_driver")
    _run([HIPCC] + SAN + ["-o", exe, stub_o] + objs)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=600)
    assert r.returncode == 0, r.stdout[-4000:]
    assert "host sanitizer driver: ok" in r.stdout
    assert "runtime error" not in r.stdout and "AddressSanitizer" not in r.stdout
