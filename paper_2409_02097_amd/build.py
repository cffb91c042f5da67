"""Builds the gfx950 shared library (and nothing else) with hipcc, in-tree.

    python -m paper_2409_02097_amd.build            # compile -> paper_2409_02097_amd/liblinfusion.so
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRCS = [os.path.join(HERE, "csrc", name) for name in ("linfusion.hip", "linfusion_wide.hip", "linfusion_bwd.hip", "linfusion_mlp.hip", "linfusion_mlph.hip", "linfusion_qv.hip", "linfusion_solo.hip", "linfusion_bwdw.hip", "lf_probe.hip")]
LIB = os.path.join(HERE, "liblinfusion.so")
OBJ_DIR = os.path.join(HERE, "_build")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "--offload-compress",   # the device images are stored compressed (the library shrinks about five-fold)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def hipcc_path() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found: the library is built with ROCm's hipcc for gfx950")


def _filtered(stderr: str) -> str:
    noise = "is not a recognized feature for this target"
    return "\n".join(l for l in stderr.splitlines() if noise not in l)


def build(verbose: bool = False, extra: list[str] | None = None) -> str:
    """Compiles the translation units side by side, then links them into the shared library."""
    hipcc = hipcc_path()
    os.makedirs(OBJ_DIR, exist_ok=True)
    procs = []
    for src in SRCS:
        obj = os.path.join(OBJ_DIR, os.path.basename(src) + ".o")
        cmd = [hipcc, *HIPCC_FLAGS, *(extra or []), "-I", os.path.join(ROOT, "include"), "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((obj, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)))
    objs = []
    for obj, pr in procs:
        _, err = pr.communicate()
        err = _filtered(err)
        if pr.returncode != 0:
            raise RuntimeError(f"hipcc failed ({pr.returncode}):\n{err}")
        if verbose and err.strip():
            print(err, flush=True)
        objs.append(obj)
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB + ".tmp"]
    if verbose:
        print(" ".join(link), flush=True)
    res = subprocess.run(link, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed ({res.returncode}):\n{_filtered(res.stderr)}")
    os.replace(LIB + ".tmp", LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, extra=sys.argv[1:]))
