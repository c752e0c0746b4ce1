"""Compiles the HIP library for gfx950 in-tree (paper_2509_19368_amd/libppsd.so)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libppsd.so")
SOURCES = [os.path.join(HERE, "csrc", "ppsd_api.hip")]
HEADERS = [os.path.join(HERE, "csrc", n) for n in ("ppsd_device.h", "ppsd_kernels.h", "ppsd_mega.h", "ppsd_prefill.h",
                                                   "ppsd_batch.h")] + [os.path.join(os.path.dirname(HERE), "include", "ppsd.h")]

HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-shared", "-fPIC",
    # keep the compiler from forming packed-fp32 instructions from scalar float code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def build_library(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-o", LIB_PATH, *SOURCES]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + res.stdout + res.stderr)
    if verbose:
        print(" ".join(cmd))
    return LIB_PATH


BENCH_PATH = os.path.join(HERE, "ppsd_kernel_bench")
BENCH_SOURCE = os.path.join(HERE, "csrc", "ppsd_kernel_bench.hip")


PREFILL_BENCH_PATH = os.path.join(HERE, "ppsd_prefill_bench")
PREFILL_BENCH_SOURCE = os.path.join(HERE, "csrc", "ppsd_prefill_bench.hip")


def _build_program(path: str, source: str, verbose: bool) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [hipcc, *flags, "-o", path, source]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + res.stdout + res.stderr)
    if verbose:
        print(" ".join(cmd))
    return path


def build_kernel_bench(verbose: bool = False) -> str:
    """The standalone kernel-level benchmark of the decode kernels (no Python at run time; used under rocprofv3 --pmc)."""
    return _build_program(BENCH_PATH, BENCH_SOURCE, verbose)


def build_prefill_bench(verbose: bool = False) -> str:
    """The standalone kernel-level benchmark of the matrix-core prefill kernels."""
    return _build_program(PREFILL_BENCH_PATH, PREFILL_BENCH_SOURCE, verbose)


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_kernel_bench(verbose=True))
    print(build_prefill_bench(verbose=True))
