"""Build libspion.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libspion.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
          # No compiler-generated packed-fp32 instructions (v_pk_add/mul/fma_f32).  The feature belongs
          # to the gfx950 pass, which honours it (a float2 fused multiply-add compiles to one
          # v_pk_fma_f32 without the flag and to two v_fma_f32 with it); hipcc also hands the flag to
          # its host pass, which prints "'-packed-fp32-ops' is not a recognized feature for this
          # target" once per source.  That line is left in the compiler output.
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# (source, extra flags).  The pattern kernels take threshold decisions in fp64 whose rounding must
# follow the sequential definition: no fused multiply-add contraction there.
SOURCES = [
    ("spion_api.hip", ["-ffp-contract=off"]),
    ("pattern_kernels.hip", ["-ffp-contract=off"]),
    ("producer_kernels.hip", []),
    # MFMA accumulators in ordinary VGPRs: the softmax between two products reads them with VALU
    # instructions, and the AGPR form costs a register copy per value per step
    ("attn_kernels.hip", ["-mllvm", "-amdgpu-mfma-vgpr-form"]),
    ("attn_bf16_kernels.hip", ["-mllvm", "-amdgpu-mfma-vgpr-form"]),
    ("attn_bwd_bf16_kernels.hip", ["-mllvm", "-amdgpu-mfma-vgpr-form"]),
]


def build(verbose: bool = False) -> str:
    """Compile every source and link the shared library; always recompiles."""
    objs = []

    def compile_one(item):
        src, extra = item
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        cmd = [HIPCC, *COMMON, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        res = subprocess.run(cmd, capture_output=True, text=True)
        err = res.stderr
        if res.returncode != 0:
            raise RuntimeError(f"hipcc failed for {src}:\n{err}")
        if verbose and err.strip():
            print(err, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
