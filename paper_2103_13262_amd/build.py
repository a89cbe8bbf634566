"""Compile the HIP sources under csrc/ for gfx950 into paper_2103_13262_amd/libmoe355.so.

hipcc cross-compiles without a GPU.  Objects go to _build/ (git-ignored); the shared
library stays in-tree next to this file so that it travels with the source tree.
"""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmoe355.so")
SOURCES = ["moe_api.hip", "gate_topk.hip", "gate_bf16.hip", "gate_dense.hip", "plan.hip", "rowmove.hip", "noalloc.hip", "ggemm_f32.hip", "ggemm_bf16_sk.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++20", "-fPIC", "-Wall",
    # packed-fp32 VALU forms are kept out of all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]
# Per-source flags.  The gate kernels carry their fp64 accumulators through loops; with the accumulators of the
# matrix instructions in the separate accumulator registers the compiler copies them to and from the ordinary
# registers around every loop iteration (and drains the matrix pipeline to do it), so for this file the matrix
# instructions are told to accumulate in ordinary registers.
SOURCE_FLAGS = {"gate_topk.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


def _compile(src):
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    cmd = [HIPCC, *FLAGS, *SOURCE_FLAGS.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the packed-fp32 feature name; that warning is harmless
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    return obj, err


def build_library(verbose=False):
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        results = list(ex.map(_compile, SOURCES))
    if verbose:
        for _, err in results:
            if err.strip():
                print(err)
    objs = [o for o, _ in results]
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB], check=True)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
