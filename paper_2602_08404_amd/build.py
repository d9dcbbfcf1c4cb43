"""Build libteam_moe.so (the C-ABI library of HIP kernels) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(CSRC, "_build")
LIB = os.path.join(HERE, "libteam_moe.so")
# (source, object suffix, extra defines); the FFN kernel file is compiled once per supported hidden size
SOURCES = [("api.hip", "", []), ("route.hip", "", []), ("dispatch.hip", "", []), ("combine.hip", "", []), ("classify.hip", "", []), ("ffn_f32.hip", "", []), ("tuning.hip", "", []), ("stream_read.hip", "", []),
           ("ffn_bf16.hip", "", [])] + [("ffn_bf16_kernel.hip", f"_ksa{ksa}", [f"-DFFN_KSA_THIS_FILE={ksa}"]) for ksa in (16, 8, 4, 2)] \
          + [("ffn_bf16_kernel.hip", f"_w8_ksa{ksa}", [f"-DFFN_KSA_THIS_FILE={ksa}", "-DFFN_W8_THIS_FILE=1"]) for ksa in (16, 8)]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed-fp32 ops are switched off for device code: some forms have produced wrong results on this hardware.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-command-line-argument",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(job) -> str:
    src, suffix, defines = job
    obj = os.path.join(OBJ, src.replace(".hip", suffix + ".o"))
    subprocess.run([HIPCC, *FLAGS, *defines, "-c", os.path.join(CSRC, src), "-o", obj], check=True)
    return obj


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
