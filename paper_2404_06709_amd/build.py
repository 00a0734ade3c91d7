"""Builds libcqil.so (gfx950) in-tree with hipcc.  Usage: python -m paper_2404_06709_amd.build

CQIL_HOST_SANITIZE=1 builds libcqil_san.so instead: the same library with AddressSanitizer + UndefinedBehaviorSanitizer
on its HOST code only (argument checks, layouts, launch set-up; the device code is unchanged), for the CPU tests of the
boundary.  The sanitizer runtime has to be in the process before python starts:
    LD_PRELOAD=$(/opt/rocm/bin/hipcc -print-file-name=libclang_rt.asan-x86_64.so) ASAN_OPTIONS=detect_leaks=0 \
        CQIL_HOST_SANITIZE=1 python -m pytest tests/test_boundary.py -m "not gpu"
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
SANITIZE = os.environ.get("CQIL_HOST_SANITIZE", "") not in ("", "0")
LIB = os.path.join(HERE, "libcqil_san.so" if SANITIZE else "libcqil.so")
SOURCES = ["cqil_host.hip", "cqil_pack.hip", "cqil_decode.hip", "cqil_generic.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-function",
    # packed fp32 instructions are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]
# host pass only: every -fsanitize= sits directly behind an -Xarch_host
SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
             "-fno-omit-frame-pointer", "-g"] if SANITIZE else []


def _compile(src: str) -> str:
    obj = os.path.join(CSRC, src.replace(".hip", "_san.o" if SANITIZE else ".o"))
    cmd = [HIPCC, *FLAGS, *SAN_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> str:
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(_compile, SOURCES))
    link_san = [*SAN_FLAGS, "-shared-libsan"] if SANITIZE else []
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *link_san, "-o", LIB, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr}")
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build()
