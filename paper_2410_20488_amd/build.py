"""Build libfirp.so for gfx950 with hipcc (in-tree, next to this file)."""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfirp.so")
SOURCES = ["engine.hip", "kernels_misc.hip", "gemm_simple.hip", "gemm_mfma.hip", "gemm_tall.hip", *[f"gemm_mfma_nw{i}.hip" for i in range(2, 9)], "attention_simple.hip", "attention_mfma.hip", "tree_search.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-Wno-pass-failed"]


def _compile(src: str) -> str:
    obj = os.path.join(HERE, "_build", src.replace(".hip", ".o"))
    os.makedirs(os.path.dirname(obj), exist_ok=True)
    cmd = ["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> str:
    with concurrent.futures.ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr}")
    # standalone per-kernel benchmark beside bench.py (links the library; the rocprofv3 counter runs use it)
    root = os.path.dirname(HERE)
    tool = os.path.join(root, "bench_projection")
    cmd = ["hipcc", *FLAGS, f"-I{CSRC}", os.path.join(root, "bench_projection.hip"), "-o", tool, f"-L{HERE}", "-lfirp",
           f"-Wl,-rpath,$ORIGIN/{os.path.basename(HERE)}"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"building bench_projection failed:\n{r.stderr}")
    if verbose:
        print(f"built {LIB} and {tool}")
    return LIB


if __name__ == "__main__":
    build()
