"""Builds liblcsa.so (gfx950 only) in-tree with hipcc.  `python -m paper_2510_12747_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblcsa.so")
SOURCES = ["lcsa_host.hip", "lcsa_pool_append.hip", "lcsa_select.hip", "lcsa_attn_generic.hip", "lcsa_attn_mfma.hip",
           "lcsa_evict.hip", "lcsa_attn_bwd.hip", "lcsa_attn_bwd_mfma.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         # packed-fp32 VALU forms are kept out of the generated code on purpose
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function"]


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *FLAGS, "-o", LIB, *[os.path.join(CSRC, s) for s in SOURCES]]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the packed-fp32 feature name and says so once per file: harmless
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return LIB


def build_bench_aids(verbose: bool = False) -> str:
    """bench.py's measurement aids (matrix-instruction loops, the attention kernel with time stamps), a shared
    object of their own."""
    root = os.path.dirname(HERE)
    out = os.path.join(root, "libbench_probe.so")
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    # the attention kernel once more, with its time stamps compiled in (the library's own copy has none)
    cmd = [hipcc, *FLAGS, "-DLCSA_TIMERS=2", "-I", root, "-o", out, os.path.join(root, "bench_probe.hip"),
           os.path.join(CSRC, "lcsa_attn_mfma.hip")]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l))
    return out


if __name__ == "__main__":
    print(build(verbose=True))
    print(build_bench_aids(verbose=True))
