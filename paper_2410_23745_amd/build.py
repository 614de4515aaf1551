"""Compile the HIP library for gfx950 in-tree: `python -m paper_2410_23745_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libsyno.so")

SOURCES = ["planner.cpp", "api.cpp", "kernels_generic.hip", "kernels_bandwidth.hip", "kernels_window.hip", "kernels_view.hip", "kernels_mfma.hip",
           "kernels_mfma_f32_lo.hip", "kernels_mfma_f32_hi.hip", "kernels_mfma_bf16_f32out.hip", "kernels_mfma_bf16_f32out_b.hip",
           "kernels_mfma_bf16_bf16out.hip", "kernels_mfma_bf16_bf16out_b.hip", "kernels_mfma_dw.hip", "conv_rows_bf16.hip", "debug_rate.hip"]

# packed-fp32 instruction selection is switched off for device code (host pass warns it does not know
# the feature; harmless)
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-command-line-argument",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _headers():
    import glob
    return glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h"))


def _compile(src: str, incremental: bool = False) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    if incremental and os.path.exists(obj):
        deps = [os.path.join(CSRC, src), os.path.abspath(__file__)] + _headers()
        if all(os.path.getmtime(d) <= os.path.getmtime(obj) for d in deps):
            return obj
    cmd = ["hipcc", "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj] + FLAGS
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(jobs: int = 8, incremental: bool = False) -> str:
    """Compiles every source (incremental: only what is older than its source or a header) and links libsyno.so."""
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda src: _compile(src, incremental), SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(incremental="--incremental" in sys.argv[1:]))
