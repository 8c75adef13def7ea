"""Build libpromptcache.so (gfx950 HIP kernels + host runtime) in-tree with hipcc.

    python -m paper_2311_04934_amd.build

hipcc cross-compiles for gfx950 without a GPU present.  Objects go to
``_build/`` (ignored by git); the shared library lands next to this file.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(ROOT, "include")
OBJDIR = os.path.join(ROOT, "_build")
LIB = os.path.join(HERE, "libpromptcache.so")

SOURCES = ["runtime.hip", "gather.hip", "rope.hip", "attn_f32.hip", "attn_bf16.hip", "attn_bf16_wide.hip", "calib.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 VALU forms
    "-Wall", "-Wno-unused-function",
    "-I", INCLUDE, "-I", CSRC,
]


def library_path() -> str:
    return LIB


def ensure_built() -> str:
    """Build only when no library is there (tests, the smoke check and the benchmark load what is built)."""
    return LIB if os.path.exists(LIB) else build()


def build(verbose: bool = False, extra_flags=()) -> str:
    os.makedirs(OBJDIR, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(OBJDIR, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [HIPCC, *FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        # hipcc's host pass does not know the device-only target feature and says so once per pass
        lines = [ln for ln in out.splitlines() if "is not a recognized feature for this target" not in ln]
        if p.returncode != 0:
            failed = True
        if lines and (verbose or p.returncode != 0 or any("warning" in ln or "error" in ln for ln in lines)):
            print(f"--- {src}\n" + "\n".join(lines), flush=True)
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
