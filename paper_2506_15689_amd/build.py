"""Builds libbasq.so (the HIP kernels and the C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
BUILD = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libbasq.so")

SOURCES = ["api.hip", "hadamard28.hip", "rotate_quant.hip", "rotate_quant_pow2.hip", "rotate_quant_k28.hip", "rotate_quant_head.hip", "rotate_quant_block.hip", "gemm_w4a4.hip", "gemm_w4a4_direct.hip", "gemm_w4a4_fp6.hip", "gemm_w4a4_grouped.hip", "gemm_w4a4_grouped_fp6.hip", "fp6_pack.hip", "gemv_w4a4.hip", "linear_decode.hip", "weights.hip", "diag.hip"]

# -ffp-contract=off: the quantiser's fp32 sequence is part of the interface; fused multiply-adds
# appear only where the source says fmaf.  Packed fp32 instructions are switched off.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _compile(src: str) -> str:
    obj = os.path.join(BUILD, os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc(), *HIPCC_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{out}")
    if out.strip():
        sys.stderr.write(out + "\n")
    return obj


def build_lib(verbose: bool = True, extra_flags=(), out: str = LIB) -> str:
    """Compile every translation unit and link libbasq.so.  Always recompiles.
    `extra_flags` (e.g. -D tuning macros) and `out` exist for tuning experiments."""
    global BUILD
    if out != LIB:
        BUILD = os.path.join(PKG, "_build", os.path.basename(out))
    os.makedirs(BUILD, exist_ok=True)
    HIPCC_FLAGS.extend(extra_flags)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-Wl,-z,defs", "-o", out, *objs]
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        raise RuntimeError("link failed:\n" + proc.stdout)
    if verbose:
        print(f"built {out}")
    return out


if __name__ == "__main__":
    # python -m paper_2506_15689_amd.build [--out path.so] [extra hipcc flags ...]
    argv = sys.argv[1:]
    out_path = LIB
    if len(argv) >= 2 and argv[0] == "--out":
        out_path, argv = os.path.abspath(argv[1]), argv[2:]
    build_lib(extra_flags=argv, out=out_path)
