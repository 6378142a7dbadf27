"""Builds liblbpwht.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

    python -m paper_2309_15275_amd.build          # compile everything, link
"""
import concurrent.futures
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
BUILD = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "liblbpwht.so")

SOURCES = ["lbp_host.cpp", "wht_kernels.hip", "wht_mfma_kernels.hip", "energy_kernels.hip", "extra_kernels.hip", "gemm_kernels.hip", "gemm_mfma.hip",
           "gemm_mfma_128x128.hip", "gemm_mfma_64x128.hip", "gemm_mfma_256x128.hip",
           "gemm_mfma_256x256.hip", "gemm_mfma_128x128w8.hip", "gemm_mfma_64x128w8.hip", "gemm_mfma_64x64.hip", "gemm_mfma_256x192.hip", "gemm_mfma_pair.hip",
           "lbp_api.hip"]

# -packed-fp32-ops off: the compiler must not form packed fp32 instructions on this target.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src):
    obj = os.path.join(BUILD, os.path.splitext(src)[0] + ".o")
    cmd = ["hipcc", "-x", "hip"] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose=True):
    """Compiles every source (always) and links the shared library.  Returns its path."""
    os.makedirs(BUILD, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=8) as pool:
        objs = list(pool.map(_compile, SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stderr)
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build()
