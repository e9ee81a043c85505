"""Build the HIP library in-tree: hipcc -> paper_2402_14160_amd/librsd.so (gfx950).

Every source is compiled to an object of its own (in parallel) and the objects are linked into
one shared library; no kernel calls device code of another file."""
import json
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "librsd.so")
RESOURCES = os.path.join(OBJ, "kernel_resources.json")
SOURCES = ["rsd_misc.hip", "vocab_kernels.hip", "rrs_kernels.hip", "tree_attention.hip", "filter_kv.hip", "prob_filter.hip", "baselines.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Rpass-analysis=kernel-resource-usage",
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
    return res.stderr


def _resource_table(remarks):
    """{kernel symbol: {"VGPRs": n, "ScratchSize": bytes per lane, ...}} from the compiler's
    kernel-resource-usage remarks."""
    table, cur = {}, None
    for line in remarks.splitlines():
        m = re.search(r"remark: (?:\s*)Function Name: (\S+)", line)
        if m:
            cur = table.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark: \s+([A-Za-z ]+?)(?: \[[^\]]*\])?: (\d+)", line)
        if m and cur is not None:
            cur[m.group(1).strip()] = int(m.group(2))
    return table


def kernel_resources():
    """Register, scratch and LDS use of every kernel as the last build() reported it."""
    with open(RESOURCES) as f:
        return json.load(f)


def build(verbose=False):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    objs = [os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES]

    def compile_one(pair):
        src, obj = pair
        return _run([hipcc] + FLAGS + EXTRA.get(src, []) + ["-c", os.path.join(CSRC, src), "-o", obj], verbose)

    with ThreadPoolExecutor(max_workers=min(4, len(SOURCES))) as pool:
        remarks = list(pool.map(compile_one, zip(SOURCES, objs)))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB], verbose)
    table = {}
    for text in remarks:
        table.update(_resource_table(text))
    with open(RESOURCES, "w") as f:
        json.dump(table, f, indent=1, sort_keys=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
