"""Compile libpab.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpab.so")
SOURCES = [os.path.join(CSRC, "pab_api.hip")]
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed fp32 VALU forms stay off for device code (the host pass does not know the
    # feature and says so; that warning is harmless)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # MFMA results feed VALU code (softmax): select the VGPR form so that no accumulator has to be
    # copied between the AGPR and VGPR halves of the register file
    "-mllvm", "-amdgpu-mfma-vgpr-form",
    # no NaN bookkeeping in max chains (masked scores are -inf, never NaN)
    "-fno-honor-nans",
    "-Wno-unused-command-line-argument",
]


def build_lib(verbose: bool = False, extra_flags=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [hipcc] + HIPCC_FLAGS + list(extra_flags) + ["-o", tmp] + SOURCES
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        sys.stderr.write(out + "\n")
        raise RuntimeError("hipcc failed building libpab.so")
    if verbose and out.strip():
        print(out)
    os.replace(tmp, LIB)
    return LIB


def ensure_built() -> str:
    """Build the library only if none is there: callers load what is built."""
    return LIB if os.path.exists(LIB) else build_lib()


def device_asm(path: str, extra_flags=()) -> str:
    """Write the gfx950 assembly of the device code (same flags as the library) to `path`."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [hipcc] + flags + list(extra_flags) + ["-S", "--cuda-device-only", "-o", path] + SOURCES
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + "\n")
        raise RuntimeError("hipcc failed writing the device assembly")
    return path


if __name__ == "__main__":
    print(build_lib(verbose=True))
