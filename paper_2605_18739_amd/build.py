"""Builds the HIP library (gfx950) in-tree: python -m paper_2605_18739_amd.build

Every source is compiled to an object of its own, side by side (the GEMM tile shapes are separate
translation units for this), and the objects are linked into libnvfp4_hip.so next to this file."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libnvfp4_hip.so")
SOURCES = ["nvfp4_gemm_tile_256x256.hip", "nvfp4_gemm_tile_256x192.hip", "nvfp4_gemm_tile_128x128.hip",
           "nvfp4_gemm_tile_64x64.hip", "nvfp4_quantize.hip", "nvfp4_quantize_resident.hip", "nvfp4_gemm.hip", "nvfp4_probe.hip", "nvfp4_api.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         # packed-FP32 instructions are kept out of every kernel
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines() if "is not a recognized feature" not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build(verbose=True):
    os.makedirs(OBJ, exist_ok=True)
    objs = [os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES]
    jobs = max(1, min(len(SOURCES), 16, int(os.environ.get("MAX_JOBS", os.cpu_count() or 4))))
    with ThreadPoolExecutor(jobs) as pool:
        list(pool.map(lambda so: _run(["hipcc"] + FLAGS + ["-c", os.path.join(CSRC, so[0]), "-o", so[1]], verbose),
                      zip(SOURCES, objs)))
    _run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB], verbose)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
