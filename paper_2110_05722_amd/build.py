"""Builds `liblsq.so` (the C-ABI library of include/lsq.h) for gfx950 with hipcc.

    python -m paper_2110_05722_amd.build

hipcc cross-compiles without a GPU.  Each translation unit is compiled on its
own (in parallel) and the objects are linked into one shared library that sits
next to this file, so it travels with the source tree.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
# LSQ_LIB_NAME / LSQ_DEFINES: build an experimental variant next to the default library (tuning only)
LIB = os.path.join(HERE, os.environ.get("LSQ_LIB_NAME", "liblsq.so"))
OBJ_DIR = os.path.join(HERE, "_build", os.environ.get("LSQ_LIB_NAME", "liblsq.so"))
SOURCES = ["api", "adam", "bias_dropout_residual", "bias_act_dropout", "heads", "embedding", "pad", "layernorm", "softmax", "ls_xent"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-command-line-argument",
    # packed fp32 VALU forms are switched off for the device pass (the host pass warns that it
    # does not know the feature; that is harmless)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
] + os.environ.get("LSQ_DEFINES", "").split()


def _compile(name: str) -> str:
    src = os.path.join(CSRC, name + ".hip")
    obj = os.path.join(OBJ_DIR, name + ".o")
    r = subprocess.run([HIPCC, *FLAGS, "-c", src, "-o", obj], capture_output=True, text=True)
    noise = ("packed-fp32-ops", "1 warning generated")
    err = "\n".join(l for l in r.stderr.splitlines() if not any(n in l for n in noise))
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {name}.hip:\n{r.stderr}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True,
                   capture_output=not verbose)
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build()
