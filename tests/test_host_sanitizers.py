"""The library's host code (configuration checks, sizes, packing, network plans, argument validation) under
AddressSanitizer and UndefinedBehaviorSanitizer: every source is compiled with `-Xarch_host -fsanitize=...` (device
code is not instrumented; GPU sanitizers are not available here) and tests/host_sanitizer_driver.cpp walks the ABI's
host-only paths.  No GPU is needed: nothing in the walk launches a kernel."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

from paper_1707_00424_amd import build as pbuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
# host pass only: the device pass of every source is compiled as always
SAN = "-Xarch_host -fsanitize=address,undefined -Xarch_host -fno-sanitize-recover=undefined -O1 -g".split()
LINK = "--offload-arch=gfx950 -fno-gpu-sanitize -fsanitize=address,undefined".split()


def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    if not os.path.exists(pbuild.HIPCC):
        pytest.skip("hipcc not found")
    flags = [f for f in pbuild.FLAGS if f != "-O3"] + SAN

    def compile_one(src):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        r = subprocess.run([pbuild.HIPCC, *flags, "-x", "hip", "-c", src, "-o", obj], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        return obj

    sources = [os.path.join(pbuild.CSRC, s) for s in pbuild.SOURCES] + [os.path.join(ROOT, "tests", "host_sanitizer_driver.cpp")]
    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(compile_one, sources))
    exe = str(tmp_path / "host_walk")
    r = subprocess.run([pbuild.HIPCC, *LINK, "-o", exe, *objs], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0 and "host walk ok" in r.stdout, (r.stdout[-1500:], r.stderr[-3000:])
