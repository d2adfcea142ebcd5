"""Builds libusv.so (HIP kernels + C ABI) for gfx950 in-tree with hipcc.  `python -m paper_2512_05754_amd.build`."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libusv.so")
SOURCES = ("usv_api.hip", "usv_scores.hip", "usv_topk.hip", "usv_attn_f32.hip", "usv_attn_bf16.hip",
           "usv_reorder.hip", "usv_coarse.hip", "usv_entropy.hip",
           "usv_merge.hip")


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found; libusv.so cannot be built")
    return exe


def build_library(verbose: bool = True, extra_flags=()) -> str:
    """Compiles every HIP source and links libusv.so.  Always recompiles."""
    cmd = [
        hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
        "-I", os.path.join(ROOT, "include"), "-I", CSRC,
        *extra_flags,
        *[os.path.join(CSRC, s) for s in SOURCES],
        "-o", LIB_PATH + ".tmp",
    ]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "'-packed-fp32-ops' is not a recognized feature"
    log = "\n".join(ln for ln in (res.stdout + res.stderr).splitlines() if noise not in ln)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + log)
    if verbose and log.strip():
        print(log)
    os.replace(LIB_PATH + ".tmp", LIB_PATH)
    return LIB_PATH


TOOLS_DIR = os.path.join(PKG_DIR, "tools")
PEAK_TOOL = os.path.join(TOOLS_DIR, "mfma_peak")


def build_tools(verbose: bool = True) -> str:
    """Compiles the stand-alone MFMA-only peak probe (measurement aid; not part of libusv.so)."""
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument", "-Wno-unused-result", os.path.join(TOOLS_DIR, "mfma_peak.hip"),
           "-o", PEAK_TOOL]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    return PEAK_TOOL


DEMO_TOOL = os.path.join(TOOLS_DIR, "usv_demo")


def build_demo(verbose: bool = True) -> str:
    """Compiles tools/usv_demo.c, a plain C99 program that drives the three stages through the C ABI, with gcc."""
    rocm = os.path.dirname(os.path.dirname(os.path.realpath(hipcc())))
    cmd = [shutil.which("gcc") or "gcc", "-std=c99", "-O2", "-Wall", "-Wextra", "-Werror", "-D__HIP_PLATFORM_AMD__",
           "-I", os.path.join(rocm, "include"), "-I", os.path.join(ROOT, "include"), os.path.join(TOOLS_DIR, "usv_demo.c"),
           "-o", DEMO_TOOL, "-L", PKG_DIR, "-l:libusv.so", "-L", os.path.join(rocm, "lib"), "-lamdhip64",
           "-Wl,-rpath,$ORIGIN/..", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("gcc failed:\n" + res.stdout + res.stderr)
    return DEMO_TOOL


if __name__ == "__main__":
    print(build_library(extra_flags=tuple(sys.argv[1:])))
    print(build_tools())
    print(build_demo())
