"""Builds the HIP library in-tree: paper_2403_09603_amd/libvt_hip.so (gfx950 only)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libvt_hip.so")
SOURCES = ["vt_gemm_shape_128x128.hip", "vt_gemm_shape_64x64.hip",
           "vt_api.hip", "vt_round_kernels.hip", "vt_round_onepass.hip", "vt_round_dense.hip", "vt_round_rowwise.hip", "vt_layers.hip", "vt_hash.hip",
           "vt_gemm_kernels.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option"] + os.environ.get("VT_EXTRA_FLAGS", "").split()


def build_lib(verbose: bool = False) -> str:
    """Compile every source for gfx950 and link the shared library. Always recompiles."""
    def compile_one(src):
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{err}")
        if verbose and err.strip():
            print(err, file=sys.stderr)
        return obj

    # the translation units are independent: compile them side by side (the GEMM tile shapes dominate)
    with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1, 8)) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose=True))
