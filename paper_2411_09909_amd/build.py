"""Builds libamxfp4.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree next to this file.

Run as `python -m paper_2411_09909_amd.build`. hipcc cross-compiles, so no GPU is needed to build.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libamxfp4.so")
SOURCES = ["api.hip", "cast.hip", "gemm_bf16.hip", "gemm_fp4.hip", "gemm_e5m2.hip", "gemm_fp8m.hip", "gemm_fp6m.hip", "layer_ops.hip", "peaks.hip", "attention.hip", "attention_decode.hip", "gemm_skinny.hip"]
# packed FP32 VALU ops are switched off on purpose (they have given wrong results on these machines)
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++20", "-fPIC", "-Wall", "-Wno-unused-command-line-argument",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src):
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    cmd = ["hipcc"] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (r.stdout + r.stderr).splitlines() if "packed-fp32-ops" not in l)
    return src, r.returncode, out, obj


def build(verbose=True):
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=4) as ex:
        results = list(ex.map(_compile, SOURCES))
    for src, rc, out, _ in results:
        if out.strip() and verbose:
            print("[%s]\n%s" % (src, out), file=sys.stderr)
        if rc:
            raise RuntimeError("hipcc failed on %s" % src)
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + [r[3] for r in results]
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build())
