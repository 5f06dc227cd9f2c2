"""Build libspecext.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libspecext.so")
# per-source extra flags: the matrix-core kernels with a softmax are compiled with the matrix-core results in
# architectural VGPRs (the softmax reads them with vector ALU instructions, which cannot read AGPRs);
# the row-split kernels never produce a NaN on their hot path, and saying so spares the max
# reductions one canonicalising instruction per operand
EXTRA_FLAGS = {"prefix_mfma.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
               "prefix_mfma_rows.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form", "-fno-honor-nans"],
               "prefill_rows.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form", "-fno-honor-nans"]}
SOURCES = ["api.hip", "prefix_generic.hip", "prefix_mfma.hip", "prefix_mfma_rows.hip", "tree_merge.hip", "retrieval.hip",
           "accept.hip", "materialized.hip", "prefill_rows.hip", "calibrate.hip"]


def hipcc_path() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", shutil.which("hipcc")):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found (set HIPCC or install ROCm under /opt/rocm)")


STAMPS_LIB_PATH = os.path.join(PKG_DIR, "libspecext_stamps.so")


def build_library(verbose: bool = True, stamps: bool = False) -> str:
    """Compile every HIP source for gfx950 and link libspecext.so next to this file.
    stamps=True builds the profiling variant libspecext_stamps.so instead (-DSPECEXT_TAIL_STAMPS: the row-split
    prefix kernel and the fused merge tail leave wall-clock stamps of their phases in the workspace; see
    paper_2505_20776_amd/phase_stamps.py)."""
    obj_dir = os.path.join(PKG_DIR, "_build_stamps" if stamps else "_build")
    os.makedirs(obj_dir, exist_ok=True)
    common = [
        hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-Wall", "-Wno-unused-function", "-Wno-inline-asm",
    ] + (["-DSPECEXT_TAIL_STAMPS"] if stamps else [])
    lib_path = STAMPS_LIB_PATH if stamps else LIB_PATH
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(obj_dir, src.replace(".hip", ".o"))
        objs.append(obj)
        procs.append((src, subprocess.Popen(common + EXTRA_FLAGS.get(src, []) + ["-c", os.path.join(CSRC, src), "-o", obj],
                                            stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for src, pr in procs:
        out, _ = pr.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if pr.returncode != 0:
            failed = True
            sys.stderr.write(f"[specext build] {src} failed:\n{out}\n")
        elif verbose and out.strip():
            sys.stderr.write(f"[specext build] {src}:\n{out}\n")
    if failed:
        raise RuntimeError("hipcc failed")
    tmp = lib_path + ".tmp"
    subprocess.run([hipcc_path(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs, check=True)
    os.replace(tmp, lib_path)
    return lib_path


if __name__ == "__main__":
    print(build_library(stamps="--stamps" in sys.argv[1:]))
