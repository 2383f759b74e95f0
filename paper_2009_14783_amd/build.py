"""Builds libhetseq_hip.so (gfx950) in-tree with hipcc.  Run: python -m paper_2009_14783_amd.build"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libhetseq_hip.so")
SOURCES = ["context.cpp", "dataset.cpp", "gemm.hip", "gemm_wide_kk.hip", "gemm_wide_kn.hip", "gemm_wide_nn.hip", "attention.hip", "attention_mfma.hip", "attention_general.hip", "rowops.hip", "seq2seq_ops.hip", "seq2seq.hip", "optim.hip", "api.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-x", "hip",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-result", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


# The wide-tile GEMM kernels unroll their epilogues over up to 16 accumulator tiles; above the compiler's default
# budget for "#pragma unroll" the loop would stay rolled and the accumulators would live in scratch memory.
EXTRA = {src: ["-mllvm", "-pragma-unroll-threshold=200000"] for src in ("gemm_wide_kk.hip", "gemm_wide_kn.hip", "gemm_wide_nn.hip")}


def _compile(src: str, objdir: str) -> str:
    obj = os.path.join(objdir, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC] + FLAGS + EXTRA.get(src, []) + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}\n{r.stderr}")
    return obj


def build(verbose: bool = True) -> str:
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda s: _compile(s, objdir), SOURCES))
    cmd = [HIPCC, "-shared", "-fPIC", "-pthread", "--offload-arch=gfx950", "-o", LIB] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
