"""Builds libhalo.so (hand-written HIP kernels for gfx950 + the C ABI) in-tree with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
INCLUDE = os.path.join(ROOT, "include")
LIB_PATH = os.path.join(PKG_DIR, "libhalo.so")
BUILD_DIR = os.path.join(PKG_DIR, "_build")

SOURCES = ["halo_api.hip", "row_transform.hip", "col_ops.hip", "gemm_i8.hip", "gemm_mx6.hip", "row_kron.hip", "lowrank.hip"]

# -ffp-contract=off: every fp32 add/mul of the rotation and the quantiser is rounded on its own, which is
# what makes the INT8 codes reproducible bit for bit.  Packed fp32 instructions are switched off.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-I" + INCLUDE, "-I" + CSRC,
]


def _hipcc() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found: libhalo needs the ROCm toolchain to build")


def _run(cmd):
    proc = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in proc.stderr.splitlines()
                    if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
    if proc.returncode != 0:
        raise RuntimeError("build step failed: %s\n%s\n%s" % (" ".join(cmd), proc.stdout, err))
    return err


def build(verbose: bool = False) -> str:
    """Compile every source for gfx950 and link libhalo.so next to this file. Always recompiles."""
    hipcc = _hipcc()
    os.makedirs(BUILD_DIR, exist_ok=True)
    objs = [os.path.join(BUILD_DIR, s.replace(".hip", ".o")) for s in SOURCES]

    def compile_one(pair):
        src, obj = pair
        return _run([hipcc, *HIPCC_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj])

    with ThreadPoolExecutor(max_workers=min(7, len(SOURCES))) as pool:
        logs = list(pool.map(compile_one, zip(SOURCES, objs)))
    logs.append(_run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB_PATH]))
    if verbose:
        for l in logs:
            if l.strip():
                print(l)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
