"""Build libfailsafe.so in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libfailsafe.so")

SOURCES = ["status.cpp", "host_builders.cpp", "host_scheduler.cpp", "host_recovery.cpp", "host_prefill.cpp", "decode_attention.hip", "merge_lse.hip", "prefill_attention.hip", "stream_probe.hip", "pack_slots.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    # keep hipcc from forming packed-fp32 instructions out of scalar float code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fvisibility=hidden",
]


def build(verbose: bool = True, extra: list[str] | None = None, out: str | None = None) -> str:
    """Compile every source into one shared library (``out``, default the in-tree libfailsafe.so)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    lib = out or LIB
    cmd = [hipcc, *FLAGS, *(extra or []), "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           "-o", lib, *[os.path.join(CSRC, s) for s in SOURCES]]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return lib


if __name__ == "__main__":
    # python -m paper_2511_14116_amd.build [-o other.so] [extra hipcc flags...]
    argv = sys.argv[1:]
    out = None
    if argv[:1] == ["-o"]:
        out, argv = argv[1], argv[2:]
    build(extra=argv, out=out)
