"""Builds the HIP library in-tree: ``python -m paper_2512_21450_amd.build``.

hipcc cross-compiles for gfx950 without a GPU.  The shared object lands next
to this file so that it travels with the source tree.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librl_decode_attn.so")
# measurement aid of bench.py (a loads-only streaming kernel), kept out of the product library
PROBE_LIB = os.path.join(HERE, "libbench_stream_read.so")
PROBE_SOURCES = ["bench_stream_read.hip"]
SOURCES = ["rlda_api.hip", "rlda_simple.hip", "rlda_shared.hip", "rlda_token_logprob.hip", "rlda_kv_append.hip",
           "rlda_policy_loss.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument"]


def _compile(out: str, sources, verbose: bool) -> None:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *FLAGS, "-o", out, *[os.path.join(CSRC, s) for s in sources]]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the packed-fp32 target feature and says so; drop that line
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed:\n{err}")
    if verbose and err.strip():
        print(err, file=sys.stderr)


def build(verbose: bool = False) -> str:
    _compile(LIB, SOURCES, verbose)
    _compile(PROBE_LIB, PROBE_SOURCES, verbose)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
