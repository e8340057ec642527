"""Builds libspa.so (gfx950 only) from csrc/*.hip with hipcc.

Usage: python -m paper_2410_23608_amd.build [--sanitize-host]
The shared library is written next to this file so that it travels with the source tree.
--sanitize-host builds libspa_asan.so in <tmp>/spa_build_asan instead: the HOST side of every source under
AddressSanitizer and UndefinedBehaviorSanitizer (device code unchanged), for the host-only checks
of tests/test_host_sanitizers.py; it is never loaded by the binding.
"""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB_PATH = os.path.join(HERE, "libspa.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=default",
    # keep the compiler from forming packed fp32 ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # MFMA accumulators in ordinary VGPRs: the softmax / rescale VALU work reads them
    # directly instead of copying through AGPRs
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",
    "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def sources():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))


# files whose kernels keep more accumulators than the ordinary half of the register file holds:
# compiled without the "MFMA results in ordinary VGPRs" option
AGPR_SOURCES = {"linear_big.hip"}


# kept out of the source tree: nothing but the host-only sanitizer test reads it
SAN_DIR = os.path.join(tempfile.gettempdir(), "spa_build_asan")
SAN_LIB_PATH = os.path.join(SAN_DIR, "libspa_asan.so")
# sanitizers on the host pass only: every -fsanitize= directly after -Xarch_host
SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
             "-fno-omit-frame-pointer", "-g"]


def _compile(src: str, sanitize: bool = False) -> str:
    obj = os.path.join(SAN_DIR if sanitize else OBJ_DIR, os.path.basename(src)[:-4] + ".o")
    flags = list(FLAGS) + (SAN_FLAGS if sanitize else [])
    if os.path.basename(src) in AGPR_SOURCES:
        i = flags.index("-amdgpu-mfma-vgpr-form=1")
        del flags[i - 1:i + 1]
    cmd = [HIPCC, *flags, "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{r.stdout}\n{r.stderr}")
    return obj


def build(verbose: bool = True, sanitize: bool = False) -> str:
    os.makedirs(SAN_DIR if sanitize else OBJ_DIR, exist_ok=True)
    srcs = sources()
    lib = SAN_LIB_PATH if sanitize else LIB_PATH
    if verbose:
        print(f"[build] compiling {len(srcs)} HIP sources for gfx950" + (" (host side sanitized)" if sanitize else ""),
              flush=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(lambda s_: _compile(s_, sanitize), srcs))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs]
    if sanitize:   # (a link line has no -Xarch_ option: the device side is kept out explicitly)
        cmd += ["-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print(f"[build] wrote {lib}", flush=True)
    return lib


def sanitized_is_current() -> bool:
    """True when the sanitized library is newer than every source and header it is built from."""
    if not os.path.exists(SAN_LIB_PATH):
        return False
    t = os.path.getmtime(SAN_LIB_PATH)
    deps = sources() + [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    deps += [os.path.join(ROOT, "include", "spa.h"), os.path.abspath(__file__)]
    return all(os.path.getmtime(d) <= t for d in deps)


if __name__ == "__main__":
    build(sanitize="--sanitize-host" in sys.argv[1:])
    sys.exit(0)
