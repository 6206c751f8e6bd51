"""Builds libdeer.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
LIB_PATH = os.path.join(PKG_DIR, "libdeer.so")
SOURCES = [os.path.join(PKG_DIR, "csrc", "deer_api.hip")]
HEADERS = [os.path.join(PKG_DIR, "csrc", "deer_kernels.hpp"), os.path.join(PKG_DIR, "csrc", "deer_tiled.hpp"), os.path.join(ROOT, "include", "deer.h")]


def hipcc_path() -> str:
    return shutil.which("hipcc") or "/opt/rocm/bin/hipcc"


def build_library(verbose: bool = False) -> str:
    """Compiles every HIP source for gfx950 and links the shared library.  Always rebuilds."""
    cmd = [
        hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
        # packed fp32 instructions are kept off for all device code
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG_DIR, "csrc"),
        "-o", LIB_PATH, *SOURCES,
    ]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)
    return LIB_PATH


def device_assembly(out_path: str) -> str:
    """The gfx950 assembly of the device code, as text (same flags as the library): for checks on the generated code."""
    cmd = [
        hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17",
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG_DIR, "csrc"),
        "--cuda-device-only", "-S", "-o", out_path, *SOURCES,
    ]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stderr)
    return out_path


if __name__ == "__main__":
    print(build_library(verbose=True))
