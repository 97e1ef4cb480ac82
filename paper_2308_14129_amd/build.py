"""Builds libtig.so (HIP, gfx950 only) in-tree with hipcc.  `python -m paper_2308_14129_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB_PATH = os.path.join(HERE, "libtig.so")
SOURCES = ["tig_api.hip", "csr_build.hip", "pack.hip", "step_launch.hip", "step_small.hip", "k_gru.hip", "k_embed.hip", "sep.hip", "pac.hip", "train.hip", "modules.hip"]

# Packed-FP32 VALU instructions are switched off for every device translation unit.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall",
               "-Wno-unused-function"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _compile(src: str, defines=(), tag: str = "") -> str:
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + tag + ".o")
    cmd = [_hipcc(), *HIPCC_FLAGS, *[f"-D{d}" for d in defines], "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


CLOCKS_LIB_PATH = os.path.join(HERE, "libtig_clocks.so")


def build(verbose: bool = False, phase_clocks: bool = False) -> str:
    """libtig.so; with phase_clocks=True instead libtig_clocks.so, the same library with per-workgroup
    timestamps at the phase boundaries of the two tile kernels (read by phase_clocks.py)."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    defines, tag, out = (("TIG_PHASE_CLOCKS",), "_clocks", CLOCKS_LIB_PATH) if phase_clocks else ((), "", LIB_PATH)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda src: _compile(src, defines, tag), SOURCES))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed:\n{res.stderr}")
    if verbose:
        print("built", out)
    return out


if __name__ == "__main__":
    build(verbose=True, phase_clocks="--phase-clocks" in sys.argv[1:])
