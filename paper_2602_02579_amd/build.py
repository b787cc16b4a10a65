"""Compile the HIP sources in ``csrc/`` into ``libpkv.so`` (gfx950 only).

``python -m paper_2602_02579_amd.build`` or ``build_library()``.  hipcc
cross-compiles without a GPU.  Objects go to ``_build/`` at the repository
root; the shared library is written next to this file so that it travels with
the source tree.
"""

from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libpkv.so")

SOURCES = ["pkv_api.hip", "rope_restore.hip", "query_score.hip", "query_score_dma.hip",
           "topk_select.hip", "gather_qkv_proj.hip", "gather_qkv_proj_dma.hip",
           "scatter_kv.hip", "layer_glue.hip", "static_scratch.hip",
           "sparse_row_attn.hip", "sparse_row_attn_dma.hip", "sparse_row_attn_w8.hip"]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument", "-Wno-inline-asm",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


# per-source additions: kernels whose MFMA results are read by the VALU right away do
# better with the results in ordinary VGPRs than with copies out of the accumulation
# registers
SOURCE_FLAGS = {
    "sparse_row_attn_dma.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
    "sparse_row_attn_w8.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
    "query_score_dma.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
}


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def build_library(verbose: bool = False, extra_flags=()) -> str:
    """Compile every source and link ``libpkv.so``; returns its path."""
    out_dir = os.path.join(ROOT, "_build")
    os.makedirs(out_dir, exist_ok=True)
    hipcc = _hipcc()

    def compile_one(src):
        obj = os.path.join(out_dir, src.replace(".hip", ".o"))
        cmd = [hipcc, *FLAGS, *SOURCE_FLAGS.get(src, ()), *extra_flags, "-c",
               os.path.join(CSRC, src), "-o", obj]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{res.stderr}")
        if verbose and res.stderr.strip():
            print(res.stderr, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    tmp = LIB_PATH + ".tmp"
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", tmp]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed:\n{res.stderr}")
    os.replace(tmp, LIB_PATH)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose="-v" in sys.argv))
