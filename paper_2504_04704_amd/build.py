"""Builds liblagkv.so (the C-ABI library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "liblagkv.so")
SOURCES = ["lagkv_api.hip", "split_pass.hip", "hold_pass.hip", "append_pass.hip", "staged_pass.hip",
           "static_scratch.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed fp32 VALU ops are kept off on this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def hipcc_path() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def _run(cmd, verbose):
    if verbose:
        print("[build]", " ".join(cmd), flush=True)
    proc = subprocess.run(cmd, capture_output=True, text=True)
    out = (proc.stdout + proc.stderr).strip()
    # the host pass does not know the gfx feature name; that warning is harmless
    out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
    if verbose and out:
        print(out, flush=True)
    if proc.returncode != 0:
        raise RuntimeError(f"hipcc failed ({proc.returncode})\n{out}")


def build_library(verbose: bool = True, extra_flags=(), out_path: str = LIB_PATH, sources=SOURCES) -> str:
    """Compile every HIP source (one hipcc process per file) and link them into
    paper_2504_04704_amd/liblagkv.so; returns its path."""
    hipcc = hipcc_path()
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    with tempfile.TemporaryDirectory(prefix="lagkv_build_") as tmp:
        objs = [os.path.join(tmp, os.path.splitext(s)[0] + ".o") for s in sources]
        cmds = [[hipcc, *HIPCC_FLAGS, *extra_flags, *inc, "-c", os.path.join(CSRC, s), "-o", o]
                for s, o in zip(sources, objs)]
        with ThreadPoolExecutor(min(len(cmds), os.cpu_count() or 1, 8)) as ex:
            list(ex.map(lambda c: _run(c, verbose), cmds))
        _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", out_path + ".tmp"], verbose)
    os.replace(out_path + ".tmp", out_path)
    return out_path


if __name__ == "__main__":
    build_library(extra_flags=sys.argv[1:])
