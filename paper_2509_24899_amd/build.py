"""Builds the C-ABI library in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_DIR = os.path.join(HERE, "lib")
LIB_PATH = os.path.join(LIB_DIR, "libhybridattn.so")
SOURCES = ["ha_api.hip", "ha_kernels.hip", "ha_state.hip", "ha_query.hip", "ha_wide.hip", "ha_wide_grad.hip", "ha_grad.hip", "ha_select.hip", "ha_update.hip"]
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
    # packed fp32 VALU forms are switched off for every device compile
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


# Per-file additions.  ha_grad.hip: its kernels run one wave per SIMD with 512 registers; selecting the matrix
# instructions in their vector-register form keeps the transient products of the feature-map recomputation out
# of the accumulator file, which the persistent partial sums fill (otherwise those are spilled to scratch and
# reloaded in every tile).
FILE_FLAGS = {"ha_grad.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"], "ha_kernels.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
              "ha_state.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


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


# Host-side sanitizer build (AddressSanitizer + UndefinedBehaviorSanitizer on the CPU code only; the device code is
# compiled as always).  The sources whose host code does real work (argument validation, workspace planning, the
# block-rate dynamic programme) are instrumented; the others are linked from the regular objects.
SANITIZED = ("ha_api.hip", "ha_select.hip")
SANITIZER_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
                   "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
SANITIZED_LIB_PATH = os.path.join(LIB_DIR, "libhybridattn_san.so")


def asan_runtime() -> str:
    """Path of the shared AddressSanitizer runtime of the compiler that hipcc drives (to be preloaded into an
    uninstrumented host program such as python)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = subprocess.run([hipcc, "-print-file-name=libclang_rt.asan-x86_64.so"], check=True, capture_output=True, text=True)
    return out.stdout.strip()


def build_sanitized_host_library() -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(LIB_DIR, exist_ok=True)
    plain = [os.path.join(LIB_DIR, s.replace(".hip", ".o")) for s in SOURCES if s not in SANITIZED]
    if not all(os.path.exists(o) for o in plain):
        build_library()
    objs, procs = list(plain), []
    for src in SANITIZED:
        obj = os.path.join(LIB_DIR, src.replace(".hip", "_san.o"))
        cmd = [hipcc, *HIPCC_FLAGS, *FILE_FLAGS.get(src, []), *SANITIZER_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for src, p in procs:
        out, _ = p.communicate()
        if p.returncode != 0:
            raise RuntimeError(f"hipcc (sanitized) failed on {src}:\n{out}")
    subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", SANITIZED_LIB_PATH], check=True)
    return SANITIZED_LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose="-v" in sys.argv))
