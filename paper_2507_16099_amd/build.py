"""Build libfp8mi355.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libfp8mi355.so")
SOURCES = ["quant_kernels.hip", "tuning.hip", "gemm_fp8.hip", "gemm_fp8_snake.hip", "gemm_fp8_stream.hip", "gemm_fp8_skinny.hip", "gemm_fp8_skinny_fused.hip", "gemm_bf16_at_b.hip", "gemm_bf16_at_b_snake.hip", "layernorm_quant.hip", "gemm_mxfp8.hip", "gemm_mxfp8_snake.hip", "api.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed-fp32 instructions are disabled on purpose (the compiler would
# otherwise form v_pk_*_f32 from plain float code)
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++20", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unknown-warning-option", "-Wno-unused-command-line-argument"]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{r.stdout}\n{r.stderr}")
    noise = ("is not a recognized feature", "warning generated", "warnings generated", "reserved registers: m0", "lds_dma16", "sn_lds_dma16", "may not be preserved", "^")
    err = "\n".join(l for l in r.stderr.splitlines()
                    if l.strip() and not any(n in l for n in noise) and not l.lstrip().startswith((":", "|")) and not l.lstrip()[:1].isdigit())
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    subprocess.run(cmd, check=True)
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build()
