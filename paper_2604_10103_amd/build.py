"""Build libhf.so (the gfx950 C-ABI library) in-tree with hipcc.

    python -m paper_2604_10103_amd.build

Cross-compiles without a GPU.  Object files go to ``_build/`` (ignored); the shared library
lands next to this file so that it travels with the source tree.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libhf.so")

SOURCES = [
    "hf_api.hip",
    "hf_state.hip",
    "hf_state_mfma.hip",
    "hf_select.hip",
    "hf_attn_generic.hip",
    "hf_attn_mfma.hip",
    "hf_attn_w64.hip",
    "hf_readout.hip",
    "hf_readout_mfma.hip",
    "hf_rope.hip",
    "hf_bwd.hip",
    "hf_bwd_mfma.hip",
    "hf_probe.hip",
]

FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
    "-fvisibility=hidden",
    "-munsafe-fp-atomics",          # hardware fp32 atomic add for the state reduction
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall",
    "-Wno-unused-function",
    "-Wno-inline-asm",               # the LDS-transfer asm names m0 as clobbered (it writes it); clang only notes that m0 is reserved
    "-I" + os.path.join(ROOT, "include"),
    "-I" + CSRC,
    "-DHF_BUILDING=1",
]


# per-source additions.  hf_attn_w64: the ILP-driven machine scheduler keeps several LDS fragment reads in
# flight ahead of the MFMAs of the flash-attention loops (the default one serialises them)
EXTRA_FLAGS = {
    "hf_attn_w64.hip": ["-mllvm", "-amdgpu-sched-strategy=iterative-ilp"],
}


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def build(verbose: bool = False, jobs: int = 8) -> str:
    out_dir = os.path.join(ROOT, "_build")
    os.makedirs(out_dir, exist_ok=True)
    cc = hipcc()
    objs = []

    def compile_one(src):
        obj = os.path.join(out_dir, src.replace(".hip", ".o"))
        cmd = [cc, *FLAGS, *EXTRA_FLAGS.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        msgs = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                         if "packed-fp32-ops" not in l and l.strip())
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}\n{r.stderr}")
        if msgs and verbose:
            print(msgs)
        return obj

    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    cmd = [cc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
