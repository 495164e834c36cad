"""Builds libdeltacnn.so for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIBDIR = os.path.join(HERE, "lib")
LIB = os.path.join(LIBDIR, "libdeltacnn.so")
SOURCES = [("ctx.hip", "ctx.o", []), ("mask_kernels.hip", "mask_kernels.o", []), ("tile_kernels.hip", "tile_kernels.o", []),
           ("conv_kernels.hip", "conv_kernels.o", []), ("layer.hip", "layer.o", []), ("net.hip", "net.o", [])]
# the MFMA convolution kernels: one object per (element type, accumulator block count), built in parallel
for _t, _tn in (("f16", "f16"), ("float", "f32")):
    for _nb in (4, 3, 2, 1):
        SOURCES.append(("conv_inst.hip", f"conv_{_tn}_nb{_nb}.o",
                        [f"-DDCNN_CONV_T={_t}", f"-DDCNN_CONV_TNAME={_tn}", f"-DDCNN_CONV_NB={_nb}"]))
FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(verbose: bool = False, jobs: int = 8) -> str:
    os.makedirs(LIBDIR, exist_ok=True)
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    extra_env = os.environ.get("DCNN_EXTRA_FLAGS", "").split()

    def compile_one(item) -> str:
        src, objname, extra = item
        obj = os.path.join(objdir, objname)
        cmd = [hipcc, *FLAGS, *extra_env, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src} {extra}:\n{err}")
        if verbose and err.strip():
            print(err, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
