"""Compile the HIP sources under csrc/ into paper_2512_03383_amd/libuniql.so (gfx950)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libuniql.so")
OBJ_DIR = os.path.join(HERE, "_build")
SOURCES = ["api.hip", "gemv.hip", "gemv_sym.hip", "gemv_bf16.hip", "gemv_bf16_sym.hip", "gemv_stream.hip", "gemv_stream_bf16.hip", "mlp_stream.hip", "mlp_stream_bf16.hip",
           "mfma_gemm.hip", "mfma_gemm_bf16.hip", "w4_dequant.hip", "w8.hip", "wbits.hip", "rope.hip", "probe.hip"]
# packed-fp32 VALU forms are switched off for every HIP translation unit
# (and the compiler's rewrite of atomics as wave-wide reductions: the one LDS counter of the streaming GEMV is
# incremented by one lane per wave, which the rewrite would wrap in a dozen extra instructions per loop body)
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-Wall",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-mllvm", "-amdgpu-atomic-optimizer-strategy=None"]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.sep not in c or os.path.exists(c)):
            return c
    return "hipcc"


def build_lib(verbose: bool = False) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    hipcc = _hipcc()

    def compile_one(src: str) -> str:
        obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
        cmd = [hipcc, *HIPCC_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        out = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                        if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed for {src}:\n{out}")
        if verbose and out.strip():
            print(out, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose=True))
