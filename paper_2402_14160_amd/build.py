"""Build the HIP library in-tree: hipcc -> paper_2402_14160_amd/librsd.so (gfx950)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librsd.so")
SOURCES = ["rsd_misc.hip", "vocab_kernels.hip", "rrs_kernels.hip", "tree_attention.hip", "filter_kv.hip", "prob_filter.hip", "baselines.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         # packed-fp32 VALU forms are kept out of the generated code
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def build(verbose=False):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("hipcc failed building librsd.so")
    if verbose and res.stderr.strip():
        sys.stderr.write(res.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
