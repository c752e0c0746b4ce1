"""Compiles the HIP library (paper_2509_19368_amd/libppsd.so) and the ppsd_cli driver program for gfx950, in-tree."""
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


CLI_PATH = os.path.join(HERE, "ppsd_cli")
CLI_SOURCE = os.path.join(HERE, "csrc", "ppsd_cli.hip")


def build_cli(verbose: bool = False) -> str:
    """ppsd_cli: a plain C++ program that drives libppsd.so through include/ppsd.h only (no Python at run
    time): the program to run under rocprofv3, and a C-side exercise of the ABI."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [hipcc, *flags, "-o", CLI_PATH, CLI_SOURCE, "-L" + HERE, "-lppsd", "-Wl,-rpath,$ORIGIN"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + res.stdout + res.stderr)
    if verbose:
        print(" ".join(cmd))
    return CLI_PATH


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_cli(verbose=True))
