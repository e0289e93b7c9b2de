"""Builds the HIP library (gfx950 only) in-tree with hipcc: libduo_verify.so (bf16 weights and KV cache) and
libduo_verify_fp16.so (the same sources compiled with DUO_FP16: IEEE fp16 instead)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libduo_verify.so")
LIB_PATH_FP16 = os.path.join(HERE, "libduo_verify_fp16.so")
SOURCES = [os.path.join(HERE, "csrc", "duo_api.hip")]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def _compile(extra, out_path: str, verbose: bool) -> str:
    cmd = [HIPCC] + FLAGS + list(extra) + SOURCES + ["-o", out_path]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "is not a recognized feature for this target" not in l)
    if verbose and out.strip():
        print(out, flush=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    return out_path


def build(verbose: bool = True) -> str:
    """Compiles both element types (in parallel); returns the path of the bf16 library."""
    with ThreadPoolExecutor(max_workers=2) as pool:
        jobs = [pool.submit(_compile, [], LIB_PATH, verbose), pool.submit(_compile, ["-DDUO_FP16"], LIB_PATH_FP16, verbose)]
        for j in jobs:
            j.result()
    return LIB_PATH


if __name__ == "__main__":
    build()
    sys.exit(0)
