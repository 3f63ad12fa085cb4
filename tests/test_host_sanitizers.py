"""The library's host code under AddressSanitizer and UndefinedBehaviorSanitizer.

Every source of the library is compiled for the host only (no device code, nothing can be
launched) with both sanitizers and linked with tests/native/host_check.cpp, which walks the
argument validation of every entry point, the partition arithmetic and the split solver (against
an exhaustive search).  A sanitizer report makes the program exit with an error."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    from paper_2009_09523_amd import build as vfbuild
    if not os.path.exists(vfbuild.HIPCC):
        pytest.skip("hipcc not available")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
    common = [vfbuild.HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-I", vfbuild.CSRC, "-I", vfbuild.INCLUDE,
              "-Wno-unused-command-line-argument", *san, "-x", "hip"]
    srcs = [os.path.join(vfbuild.CSRC, f) for f in vfbuild.sources()] + [os.path.join(ROOT, "tests", "native", "host_check.cpp")]

    def compile_one(src):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        r = subprocess.run([*common, "-c", src, "-o", obj], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-3000:]
        return obj
    with ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(compile_one, srcs))
    exe = str(tmp_path / "host_check")
    r = subprocess.run([vfbuild.HIPCC, "--offload-arch=gfx950", *san, "-o", exe, *objs], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, (r.stdout[-3000:], r.stderr[-3000:])
    assert "host checks ok" in r.stdout
