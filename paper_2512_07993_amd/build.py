"""Builds libskipkv.so for gfx950 with hipcc (cross-compiles without a GPU).

    python -m paper_2512_07993_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libskipkv.so")
SOURCES = ["api.hip", "plan.hip", "scan.hip", "scan_fused.hip", "cosine.hip", "select.hip", "tokred.hip", "compact.hip", "steer.hip", "ranges.hip", "hidden.hip", "paged.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                    if "is not a recognized feature for this target" not in l)
    if r.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), out))
    return out


def build_library(verbose: bool = False, jobs: int = 8) -> str:
    hipcc = _hipcc()
    bdir = os.path.join(PKG, "_build")
    os.makedirs(bdir, exist_ok=True)
    objs = [os.path.join(bdir, s.replace(".hip", ".o")) for s in SOURCES]

    def one(pair):
        src, obj = pair
        return _run([hipcc, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj])

    with ThreadPoolExecutor(max_workers=jobs) as ex:
        outs = list(ex.map(one, zip(SOURCES, objs)))
    outs.append(_run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]))
    if verbose:
        for o in outs:
            if o.strip():
                print(o)
    return LIB


HOSTSAN_LIB = os.path.join(PKG, "_build", "libskipkv_hostsan.so")
# host side only (-Xarch_host): the device code is compiled as always.  Trap mode needs no sanitizer
# runtime, so the library loads into an ordinary Python process; undefined behaviour ends in SIGILL.
HOSTSAN_FLAGS = ["-Xarch_host", "-fsanitize=undefined,float-divide-by-zero,implicit-integer-truncation",
                 "-Xarch_host", "-fsanitize-trap=all"]


def build_host_sanitized() -> str:
    """A second library whose host side of the ABI (argument validation, workspace carving: api.hip) is
    compiled at -O1 with the undefined-behaviour sanitizer; the other objects are those of the normal
    build.  Used by tests/test_abi_sanitized.py on the CPU; never shipped, never loaded by the binding."""
    hipcc = _hipcc()
    bdir = os.path.join(PKG, "_build")
    objs = [os.path.join(bdir, s.replace(".hip", ".o")) for s in SOURCES]
    if not all(os.path.exists(o) for o in objs):
        build_library()
    san = os.path.join(bdir, "api_hostsan.o")
    flags = [f for f in FLAGS if f != "-O3"]
    _run([hipcc, *flags, "-O1", "-g", *HOSTSAN_FLAGS, "-c", os.path.join(CSRC, "api.hip"), "-o", san])
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", HOSTSAN_LIB, san, *objs[1:]])
    return HOSTSAN_LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
    sys.exit(0)
