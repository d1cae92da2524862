"""Build the C-ABI library paper_2411_00915_amd/liblora_amd.so for gfx950.

hipcc cross-compiles without a GPU.  The packed-fp32 VALU forms are switched
off for all device code (some of their forms have produced wrong results on the
target machines).
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "liblora_amd.so")
OBJ_DIR = os.path.join(HERE, "_build")

SOURCES = ["planner.cpp", "kernels_general.hip", "kernels_tiled.hip", "kernels_stream.hip", "kernels_gemm.hip", "abi.hip", "timing.hip"]

HIP_FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-Wall", "-Wno-unused-function",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
HOST_FLAGS = ["-O2", "-std=c++17", "-fPIC", "-Wall"]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ_DIR, src + ".o")
    path = os.path.join(CSRC, src)
    if src.endswith(".hip"):
        cmd = ["hipcc", "-c", path, "-o", obj] + HIP_FLAGS
    else:
        cmd = ["g++", "-c", path, "-o", obj] + HOST_FLAGS
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"compile failed: {' '.join(cmd)}\n{res.stdout}\n{res.stderr}")
    noise = "'-packed-fp32-ops' is not a recognized feature"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l).strip()
    if err:
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = ["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", OUT] + objs
    subprocess.check_call(cmd)
    if verbose:
        print(OUT)
    return OUT


if __name__ == "__main__":
    build(verbose=True)
