"""Builds libds.so (the C-ABI library) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libds.so")
SOURCES = ["ds_api.hip", "layernorm.hip", "kv_cache.hip", "gemm.hip", "gemm_skinny.hip",
           "attn_prefill.hip", "attn_decode.hip", "token_io.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


DEV_LIB_PATH = os.path.join(PKG_DIR, "libds_dev.so")


def build_library(verbose: bool = False, jobs: int = 8, dev: bool = False) -> str:
    """Compile every kernel source and link libds.so.  Always recompiles.

    dev=True builds libds_dev.so instead: the same sources with -DDS_DEV_SWITCHES, in which the planning
    choices (tile shape, split count, column cut, kernel family) can be forced at run time through
    ds_dev_switch.  Only the sweep harness (plan_sweep.py) loads it; the product never does."""
    obj_dir = os.path.join(PKG_DIR, "_build_dev" if dev else "_build")
    lib_path = DEV_LIB_PATH if dev else LIB_PATH
    flags = FLAGS + (["-DDS_DEV_SWITCHES"] if dev else [])
    os.makedirs(obj_dir, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(obj_dir, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [HIPCC, *flags, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        while sum(p.poll() is None for _, p in procs) >= jobs:
            procs[0][1].wait()
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        lines = [l for l in out.splitlines() if "not a recognized feature" not in l]
        if p.returncode != 0:
            failed = True
            print(f"--- {src} FAILED\n" + "\n".join(lines), file=sys.stderr)
        elif verbose and lines:
            print(f"--- {src}\n" + "\n".join(lines))
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib_path, *objs]
    subprocess.run(cmd, check=True)
    return lib_path


if __name__ == "__main__":
    print(build_library(verbose=True, dev="--dev" in sys.argv[1:]))
