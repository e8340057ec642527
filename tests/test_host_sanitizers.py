"""Host side of libspa under AddressSanitizer + UndefinedBehaviorSanitizer (no GPU): option parsing,
workspace queries and the argument validation of the entry points.  The sanitized build
(`python -m paper_2410_23608_amd.build --sanitize-host`, host pass only) and the driver
tests/host_sanitizer_driver.cpp are compiled on demand; the driver runs as a child process."""
import os
import shutil
import subprocess

import pytest

from paper_2410_23608_amd import build as spa_build

HERE = os.path.dirname(os.path.abspath(__file__))
CLANGXX = "/opt/rocm/lib/llvm/bin/clang++"


@pytest.mark.skipif(not (os.path.exists(spa_build.HIPCC) and os.path.exists(CLANGXX)), reason="needs hipcc and its clang++")
def test_host_side_under_asan_and_ubsan(tmp_path):
    if not spa_build.sanitized_is_current():
        spa_build.build(verbose=False, sanitize=True)
    lib_dir = spa_build.SAN_DIR
    exe = str(tmp_path / "host_sanitizer_driver")
    cmd = [CLANGXX, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-omit-frame-pointer",
           "-fno-sanitize-recover=undefined", "-I", os.path.join(spa_build.ROOT, "include"),
           os.path.join(HERE, "host_sanitizer_driver.cpp"), "-L", lib_dir, "-lspa_asan", f"-Wl,-rpath,{lib_dir}",
           "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-4000:]
    env = dict(os.environ)
    # leaks are not checked: the HIP runtime that the library links against keeps its own allocations
    # until exit; every other report ends the process with a non-zero code
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    out = r.stdout + r.stderr
    assert r.returncode == 0, out[-6000:]
    assert "host sanitizer driver: ok" in out
    assert "AddressSanitizer" not in out and "runtime error" not in out, out[-6000:]
    shutil.rmtree(tmp_path, ignore_errors=True)
