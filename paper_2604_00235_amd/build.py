"""Builds libmacattn.so (HIP kernels + C ABI) and libmacprobe.so (the read-only streaming probe bench.py uses as a
measured ceiling) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "libmacattn.so")
PROBE_LIB_PATH = os.path.join(_HERE, "libmacprobe.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def hipcc_path() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def _compile(source: str, target: str, verbose: bool, extra_flags=()) -> str:
    cmd = [hipcc_path(), *HIPCC_FLAGS, *extra_flags, os.path.join(CSRC, source), "-o", target]
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return target


def build_library(verbose: bool = False, extra_flags=()) -> str:
    """Compile csrc/mac_attn.hip into libmacattn.so (and csrc/stream_probe.hip into libmacprobe.so) next to this file
    and return the path of the former."""
    _compile("stream_probe.hip", PROBE_LIB_PATH, verbose)
    return _compile("mac_attn.hip", LIB_PATH, verbose, extra_flags)


if __name__ == "__main__":
    print(build_library(verbose=True))
