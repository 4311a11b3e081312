"""Compiles the HIP sources under `csrc/` into `libsig.so` next to this file (gfx950 only)."""
from __future__ import annotations

import concurrent.futures
import glob
import os
import shutil
import subprocess
import tempfile

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
INCLUDE = os.path.join(ROOT, "include")
LIB_PATH = os.path.join(PKG_DIR, "libsig.so")
PEAKS_SRC = os.path.join(PKG_DIR, "peaks", "peak_probe.hip")
PEAKS_LIB_PATH = os.path.join(PKG_DIR, "libsig_peaks.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
    "-Wall",
    # packed-FP32 instructions are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # keep matrix-core operands and results in ordinary vector registers: the kernels chain the
    # result of one outer product into the operand of the next, and the AGPR form costs copies
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",
]


def sources() -> list[str]:
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build_lib(verbose: bool = False, jobs: int = 8) -> str:
    """Compiles every `csrc/*.hip` (up to `jobs` at a time) and links them; returns the path of the shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = tempfile.mkdtemp(prefix="libsig_build_")
    try:
        def compile_one(src: str) -> str:
            obj = os.path.join(objdir, os.path.basename(src) + ".o")
            cmd = [hipcc, *HIPCC_FLAGS, "-I", INCLUDE, "-I", CSRC, "-c", src, "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            res = subprocess.run(cmd, capture_output=True, text=True)
            if res.returncode != 0:
                raise RuntimeError(f"hipcc failed on {src}:\n{res.stdout}\n{res.stderr}")
            if verbose and res.stderr.strip():
                print(res.stderr)
            return obj

        with concurrent.futures.ThreadPoolExecutor(max_workers=max(1, jobs)) as pool:
            objects = list(pool.map(compile_one, sources()))
        tmp = LIB_PATH + f".tmp{os.getpid()}"
        cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objects]
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError(f"link failed:\n{res.stdout}\n{res.stderr}")
        os.replace(tmp, LIB_PATH)
    finally:
        shutil.rmtree(objdir, ignore_errors=True)
    return LIB_PATH


def build_peaks_lib(verbose: bool = False) -> str:
    """Compiles the microbenchmarks of the device limits (`peaks/peak_probe.hip`, used by bench.py only) into
    `libsig_peaks.so`; returns its path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = PEAKS_LIB_PATH + f".tmp{os.getpid()}"
    flags = [f for f in HIPCC_FLAGS if f not in ("-mllvm", "-amdgpu-mfma-vgpr-form=1")]
    cmd = [hipcc, *flags, "-I", INCLUDE, "-shared", PEAKS_SRC, "-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {PEAKS_SRC}:\n{res.stdout}\n{res.stderr}")
    os.replace(tmp, PEAKS_LIB_PATH)
    return PEAKS_LIB_PATH


if __name__ == "__main__":
    print(build_lib(verbose=True))
    print(build_peaks_lib(verbose=True))
