"""Builds liblss_attn.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

    python -m paper_2311_02382_amd.build                # the library
    python -m paper_2311_02382_amd.build --microbench   # also lss_microbench (issue-rate microbenchmarks, a stand-alone program)

hipcc cross-compiles without a GPU.  The library lands next to this file so that it
travels with the source tree; nothing is installed.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

PKG = Path(__file__).resolve().parent
CSRC = PKG / "csrc"
INCLUDE = PKG.parent / "include"
LIB = PKG / "liblss_attn.so"
OBJ_DIR = PKG / "_build"

SOURCES = ["lss_fwd.hip", "lss_fwd_bf16.hip", "lss_bwd.hip", "lss_bwd_bf16.hip", "lss_reduce.hip", "lss_proj.hip", "lss_rows.hip", "lss_timing.hip", "lss_api.hip"]
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
    # keep the compiler from forming packed-fp32 VALU ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # matrix-instruction results stay in ordinary VGPRs (the softmax reads them with vector ALU
    # ops); accumulation-only registers may still be placed in the AGPR half
    "-mllvm", "-amdgpu-mfma-vgpr-form",
]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _compile(src: str) -> Path:
    obj = OBJ_DIR / (Path(src).stem + ".o")
    cmd = [_hipcc(), *HIPCC_FLAGS, f"-I{INCLUDE}", f"-I{CSRC}", "-c", str(CSRC / src), "-o", str(obj)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{r.stderr}")
    return obj


def build_library(verbose: bool = True) -> Path:
    """Compile every HIP source and link liblss_attn.so.  Always recompiles."""
    OBJ_DIR.mkdir(exist_ok=True)
    with ThreadPoolExecutor(max_workers=4) as pool:
        objs = list(pool.map(_compile, SOURCES))
    tmp = LIB.with_suffix(f".so.tmp{os.getpid()}")
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(tmp), *map(str, objs)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr}")
    os.replace(tmp, LIB)
    if verbose:
        print(f"built {LIB} ({LIB.stat().st_size} bytes)")
    return LIB


MICROBENCH = PKG / "lss_microbench"


def build_microbench(verbose: bool = True) -> Path:
    """Compile csrc/lss_microbench.hip into the stand-alone program lss_microbench."""
    cmd = [_hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-mllvm", "-amdgpu-mfma-vgpr-form", str(CSRC / "lss_microbench.hip"), "-o", str(MICROBENCH)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on lss_microbench.hip:\n{r.stderr}")
    if verbose:
        print(f"built {MICROBENCH}")
    return MICROBENCH


if __name__ == "__main__":
    build_library()
    if "--microbench" in sys.argv[1:]:
        build_microbench()
    sys.exit(0)
