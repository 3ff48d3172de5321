"""Builds libenergon.so (hand-written HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libenergon.so")
OBJ_DIR = os.path.join(os.path.dirname(PKG), "_build")

SOURCES = ["energon_api.hip", "pack.hip", "layernorm.hip", "gemm_f32.hip", "gemm_mfma.hip",
           "attention_f32.hip", "attention_mfma.hip", "drce.hip", "ln_fold.hip", "gemm_skinny.hip",
           "decode_attention.hip", "model_ends.hip"]
# packed-fp32 instructions are switched off for every device pass
FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-command-line-argument",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("command failed: %s\n%s\n%s" % (" ".join(cmd), r.stdout, err))
    return err


def build(verbose: bool = False, jobs: int = 8) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    objs = [os.path.join(OBJ_DIR, s.replace(".hip", ".o")) for s in SOURCES]

    def compile_one(pair):
        src, obj = pair
        return _run([hipcc, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj])

    with ThreadPoolExecutor(max_workers=min(jobs, len(SOURCES))) as ex:
        for src, warn in zip(SOURCES, ex.map(compile_one, zip(SOURCES, objs))):
            if verbose and warn.strip():
                print(f"[{src}]\n{warn}", file=sys.stderr)
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
