"""Builds libspectree.so (HIP kernels + C ABI) and libspecprobe.so (the read-stream measurement aid the
benchmark times beside the kernels) for gfx950 with hipcc, in-tree.

    python -m paper_2305_09781_amd.build        # compile every source, link the shared libraries
"""
from __future__ import annotations

import concurrent.futures
import os
import shutil
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
OBJ_DIR = os.path.join(PKG_DIR, "_build")
LIB_DIR = os.path.join(PKG_DIR, "lib")
LIB_PATH = os.path.join(LIB_DIR, "libspectree.so")
PROBE_LIB_PATH = os.path.join(LIB_DIR, "libspecprobe.so")

SOURCES = ["spec_api.hip", "kv_cache.hip", "tree_attention_f32.hip", "tree_attention_bf16.hip",
           "tree_attention_bf16_wide.hip", "tree_attention_bf16_wide32.hip", "verify.hip", "tree_build.hip", "lm_head.hip"]
PROBE_SOURCES = ["probe.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=fast",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-unknown-attributes",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: the HIP toolchain is required to build libspectree")
    return exe


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("command failed: %s\n%s\n%s" % (" ".join(cmd), r.stdout, r.stderr))
    noise = "'-packed-fp32-ops' is not a recognized feature"
    err = "\n".join(ln for ln in r.stderr.splitlines() if noise not in ln).strip()
    if err:
        sys.stderr.write(err + "\n")


def build_library(extra_flags=(), verbose: bool = True) -> str:
    """Compiles every source and links the shared library; returns its path."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    os.makedirs(LIB_DIR, exist_ok=True)
    hipcc = _hipcc()
    objs = []
    jobs = []
    probe_objs = []
    for src in SOURCES + PROBE_SOURCES:
        obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
        (probe_objs if src in PROBE_SOURCES else objs).append(obj)
        jobs.append([hipcc, *HIPCC_FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj])
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(jobs))) as ex:
        list(ex.map(_run, jobs))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH, *objs])
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", PROBE_LIB_PATH, *probe_objs])
    if verbose:
        print("built", LIB_PATH, "and", PROBE_LIB_PATH)
    return LIB_PATH


if __name__ == "__main__":
    build_library(extra_flags=sys.argv[1:])
