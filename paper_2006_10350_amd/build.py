"""Builds libknm.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libknm.so")
SOURCES = ["knm_tile.hip", "knm_tile_f16.hip", "knm_gemm.hip", "knm_gemm_f16.hip", "knm_api.hip", "knm_solver.hip", "knm_dsyrk.hip", "knm_sparse.hip", "knm_probe.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    # packed fp32 VALU forms are kept out of generated code on this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
    "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes", "-Wno-pass-failed",
]
# per-source extras
EXTRA = {
    # keep MFMA accumulators in architectural VGPRs so the VALU reads them without copies
    "knm_tile.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
    "knm_tile_f16.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
    # its builtin MFMAs (the reduction against the vectors) accumulate in VGPRs; the AGPRs are
    # taken by the inline-assembly accumulators of the cross term
    "knm_gemm_f16.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
    # 128 accumulator registers per wavefront, read and written by the epilogue
    "knm_dsyrk.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
}


def _compile(src: str, extra) -> str:
    obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC, *FLAGS, *EXTRA.get(src, []), *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError(f"hipcc failed on {src}")
    warn = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if warn:
        sys.stderr.write(warn + "\n")
    return obj


def build(extra_flags=(), verbose: bool = False) -> str:
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(lambda s: _compile(s, list(extra_flags)), SOURCES))
    cmd = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *objs,
           "-L/opt/rocm/lib", "-Wl,-rpath,/opt/rocm/lib"]
    subprocess.run(cmd, check=True)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(sys.argv[1:], verbose=True)
