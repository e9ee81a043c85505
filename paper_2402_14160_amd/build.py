"""Build the HIP library in-tree: hipcc -> paper_2402_14160_amd/librsd.so (gfx950).

Every source is compiled to an object of its own (in parallel) and the objects are linked into
one shared library; no kernel calls device code of another file."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "librsd.so")
SOURCES = ["rsd_misc.hip", "vocab_kernels.hip", "rrs_kernels.hip", "tree_attention.hip", "filter_kv.hip", "prob_filter.hip", "baselines.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         # packed-fp32 VALU forms are kept out of the generated code
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]
# The work-queue counter of the verification pass is read by one thread and its value is needed a
# whole group later.  The compiler's wave-level rewrite of uniform atomics puts a lane read, and
# with it a wait for every load in flight, right behind the atomic: switched off for that file.
EXTRA = {"rrs_kernels.hip": ["-mllvm", "-amdgpu-atomic-optimizer-strategy=None"]}


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("hipcc failed building librsd.so")
    if verbose and res.stderr.strip():
        sys.stderr.write(res.stderr)


def build(verbose=False):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    objs = [os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES]

    def compile_one(pair):
        src, obj = pair
        _run([hipcc] + FLAGS + EXTRA.get(src, []) + ["-c", os.path.join(CSRC, src), "-o", obj], verbose)

    with ThreadPoolExecutor(max_workers=min(4, len(SOURCES))) as pool:
        list(pool.map(compile_one, zip(SOURCES, objs)))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB], verbose)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
