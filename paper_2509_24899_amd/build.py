"""Builds the C-ABI library in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_DIR = os.path.join(HERE, "lib")
LIB_PATH = os.path.join(LIB_DIR, "libhybridattn.so")
SOURCES = ["ha_api.hip", "ha_kernels.hip", "ha_query.hip", "ha_wide.hip", "ha_wide_grad.hip", "ha_grad.hip", "ha_select.hip", "ha_update.hip"]
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
    # packed fp32 VALU forms are switched off for every device compile
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


# Per-file additions.  ha_grad.hip: its kernels run one wave per SIMD with 512 registers; selecting the matrix
# instructions in their vector-register form keeps the transient products of the feature-map recomputation out
# of the accumulator file, which the persistent partial sums fill (otherwise those are spilled to scratch and
# reloaded in every tile).
FILE_FLAGS = {"ha_grad.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"], "ha_kernels.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


def build_library(verbose: bool = False, extra_flags=(), out_path: str = LIB_PATH, tag: str = "") -> str:
    """Compile every source and link the shared library (libhybridattn.so by default); returns its path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(LIB_DIR, exist_ok=True)
    objs, procs = [], []
    for src in SOURCES:
        obj = os.path.join(LIB_DIR, src.replace(".hip", tag + ".o"))
        cmd = [hipcc, *HIPCC_FLAGS, *FILE_FLAGS.get(src, []), *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l and l.strip())
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and out:
            print(out, flush=True)
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", out_path]
    subprocess.run(link, check=True)
    return out_path


if __name__ == "__main__":
    print(build_library(verbose="-v" in sys.argv))
