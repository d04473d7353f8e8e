"""Build libtablecache.so in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtablecache.so")
SOURCES = ["tc_host.hip", "kv_stitch.hip", "prefill_attn_bf16.hip", "prefill_attn_f32.hip", "decode_attn_bf16.hip", "prefill_attn_pp_bf16.hip",
           "frontend.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 instructions
         "-Wno-unused-command-line-argument"]


def build_library(verbose: bool = True, extra_flags=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + ".%d.tmp" % os.getpid()
    cmd = [hipcc] + FLAGS + list(extra_flags) + ["-I", os.path.join(HERE, "..", "include"), "-o", tmp] + \
          [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    build_library(extra_flags=sys.argv[1:])
