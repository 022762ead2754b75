"""Builds the C-ABI shared library (gfx950 only) in-tree with hipcc.

    python -m paper_2512_12928_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_NAME = "libproserve_mi355x.so"
LIB_PATH = os.path.join(HERE, LIB_NAME)
SOURCES = ["ps_api.hip", "ps_kernels.hip", "ps_fused.hip", "ps_sched.cpp"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # keep the compiler from forming packed-fp32 VALU ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def build(verbose: bool = True) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return LIB_PATH


PROBE_PATH = os.path.join(HERE, "ps_machine_probe")


def build_probe(verbose: bool = True) -> str:
    """The stand-alone machine probe (csrc/ps_machine_probe.hip): matrix-pipe rate and shader clock against operand
    bits, cache-streaming rate per CU, and both kinds of waves on one CU.  Run it on the GPU machine as
    paper_2512_12928_amd/ps_machine_probe [mfma|stream|share]."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wall", os.path.join(CSRC, "ps_machine_probe.hip"), "-o", PROBE_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return PROBE_PATH


def build_host_checks(out_path: str, driver: str, verbose: bool = False) -> str:
    """CPU build of the whole library plus a driver program with AddressSanitizer and UndefinedBehaviorSanitizer on the
    host code (the device code is compiled as usual and never runs): for the host logic -- the batch former, the launch
    planners, the validation paths.  Returns the executable's path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = ["--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fno-omit-frame-pointer", "-Xclang", "-target-feature", "-Xclang",
             "-packed-fp32-ops", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
             "-fno-sanitize-recover=undefined", "-I", os.path.join(os.path.dirname(HERE), "include")]
    cmd = [hipcc] + flags + [driver] + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", out_path]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l))
    return out_path


if __name__ == "__main__":
    build()
    print("built", LIB_PATH)
    build_probe()
    print("built", PROBE_PATH)
    sys.exit(0)
