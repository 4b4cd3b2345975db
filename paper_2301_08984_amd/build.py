"""Builds libss_attn.so (HIP kernels + C ABI) for gfx950, in-tree.

    python -m paper_2301_08984_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libss_attn.so")
SOURCES = ["api.hip", "generic_kernels.hip", "mfma_kernels.hip", "small_kernels.hip", "fast_fwd.hip", "fast_fwd128.hip", "fast_dq.hip", "fast_rdq.hip", "fast_dq128.hip", "fast_kv128.hip", "fast_wave_fwd.hip", "fast_wave_fwd128.hip", "fast_wave_bwd.hip", "fast_wave_bwd128.hip", "ffn_kernels.hip", "ffn_api.hip", "planner.hip",
           "fast_dkdv.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


# Sources that use no accumulation registers: matrix instructions in their vector-register form, so
# that all of a wavefront's registers are vector registers (see the header of fast_wave_fwd128.hip).
VGPR_FORM = ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]
EXTRA_FLAGS = {"fast_fwd128.hip": VGPR_FORM, "fast_dq128.hip": VGPR_FORM, "fast_kv128.hip": VGPR_FORM, "fast_wave_fwd128.hip": VGPR_FORM, "fast_wave_bwd128.hip": VGPR_FORM}


def _compile(src: str, objdir: str) -> str:
    obj = os.path.join(objdir, src.replace(".hip", ".o"))
    cmd = ["hipcc", *FLAGS, *EXTRA_FLAGS.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> str:
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(lambda s: _compile(s, objdir), SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build()
