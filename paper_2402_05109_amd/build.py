"""Builds libhydra.so (gfx950) in-tree with hipcc.  `python -m paper_2402_05109_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libhydra.so")
OBJ_DIR = os.path.join(HERE, "_build")

SOURCES = ["api.hip", "glue.hip", "draft_accept.hip", "f32_family.hip", "bf16_gemm.hip", "bf16_attn.hip", "bf16_layers.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError("command failed: " + " ".join(cmd) + "\n" + r.stdout + err)
    if err.strip():
        sys.stderr.write(err + "\n")


def build_library(verbose: bool = True) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    hipcc = _hipcc()
    objs = [os.path.join(OBJ_DIR, s.replace(".hip", ".o")) for s in SOURCES]

    def one(i):
        _run([hipcc, *FLAGS, "-c", os.path.join(CSRC, SOURCES[i]), "-o", objs[i]])
        if verbose:
            print("compiled", SOURCES[i], flush=True)

    with ThreadPoolExecutor(max_workers=min(7, os.cpu_count() or 1)) as ex:
        list(ex.map(one, range(len(SOURCES))))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", OUT, *objs])
    if verbose:
        print("linked", OUT, flush=True)
    return OUT


if __name__ == "__main__":
    build_library()
