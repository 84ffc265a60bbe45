"""Builds the HIP library in-tree: paper_2602_19128_amd/libmoe_gfx950.so.

    python -m paper_2602_19128_amd.build            # the library and the streaming probe
    python -m paper_2602_19128_amd.build --probe    # the streaming probe only

Every csrc/*.hip file is one translation unit; they are compiled side by side and linked
into one shared object that exports the C ABI of include/moe.h and nothing else.
probe/stream_probe.hip is a stand-alone program (the chip's streaming-read rate with the
grouped GEMMs' access pattern); nothing in the library, the tests or the benchmark needs it.
"""
from __future__ import annotations

import concurrent.futures
import glob
import os
import shutil
import subprocess
import sys
import tempfile

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libmoe_gfx950.so")
PROBE_SRC = os.path.join(PKG, "probe", "stream_probe.hip")
PROBE = os.path.join(PKG, "probe", "stream_probe")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-fvisibility=hidden",                                          # only MOE_API symbols leave the library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 code generation
    "-Wall", "-Wno-unused-function",
    "-Wno-inline-asm",      # clang notes that the m0 clobber of the LDS-copy statements names a reserved register: intended
]
# the host pass reports the device-only target feature as unknown; that line is noise
_NOISE = "is not a recognized feature for this target"


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if _NOISE not in l)
    if err.strip() and verbose:
        print(err, file=sys.stderr)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}): {' '.join(cmd)}\n{err}")


def build_probe(verbose: bool = True) -> str:
    """Compile the stand-alone streaming probe for gfx950."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIPCC_FLAGS if f not in ("-fPIC", "-fvisibility=hidden")]
    _run([hipcc, *flags, "-o", PROBE, PROBE_SRC], verbose)
    return PROBE


def build(verbose: bool = True, jobs: int = 0) -> str:
    """Compile every HIP source for gfx950 and link the shared library (always rebuilds)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    srcs = sources()
    jobs = jobs or min(len(srcs), max(1, min(16, os.cpu_count() or 1)))
    tmp = tempfile.mkdtemp(prefix="moe_build_")
    try:
        objs = [os.path.join(tmp, os.path.basename(s)[:-4] + ".o") for s in srcs]
        with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as pool:
            futs = [pool.submit(_run, [hipcc, *HIPCC_FLAGS, *inc, "-c", s, "-o", o], verbose)
                    for s, o in zip(srcs, objs)]
            for f in futs:
                f.result()
        _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], verbose)
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
    build_probe(verbose)
    return LIB


if __name__ == "__main__":
    print(build_probe() if "--probe" in sys.argv[1:] else build())
