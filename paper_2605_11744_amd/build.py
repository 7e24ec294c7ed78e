"""Builds libsegattn.so (HIP, gfx950) in-tree with hipcc.  No fallback: the library is the product."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libsegattn.so")
SOURCES = ("segattn_api.hip", "segattn_prefill_mfma.hip", "segattn_prefill_fp32.hip", "segattn_decode.hip", "segattn_decode_mfma.hip",
           "segattn_cache.hip", "segattn_bwd_fp32.hip", "segattn_bwd_dq.hip", "segattn_bwd_mfma.hip", "segattn_rope.hip", "segattn_retrieve.hip", "segattn_probe.hip")
HIPCC_FLAGS = (
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    # packed fp32 VALU forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
)
# Per-source extras.  The forward prefill kernel and both backward kernels are built with the
# VGPR form of the matrix products: a product delivers its result in vector registers, where the
# softmax / dS arithmetic reads it, instead of in accumulation registers that have to be copied
# out first.  The forward and dQ kernels fit 256 vector registers per wave (two waves per SIMD);
# the dK/dV kernel keeps its K and V operands in accumulation registers, which the products can
# read directly.  Every other file keeps the compiler's default form.
_VGPR_FORM = ("-mllvm", "-amdgpu-mfma-vgpr-form=1")
EXTRA_FLAGS = {"segattn_prefill_mfma.hip": _VGPR_FORM, "segattn_bwd_dq.hip": _VGPR_FORM,
               "segattn_bwd_mfma.hip": _VGPR_FORM}


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: libsegattn cannot be built")
    return exe


def build(verbose: bool = False) -> str:
    """Compile every HIP source for gfx950 and link libsegattn.so.  Always recompiles."""
    objs = []
    build_dir = os.path.join(PKG_DIR, "_build")
    os.makedirs(build_dir, exist_ok=True)
    procs = []
    for src in SOURCES:
        obj = os.path.join(build_dir, src.replace(".hip", ".o"))
        cmd = [hipcc(), *HIPCC_FLAGS, *EXTRA_FLAGS.get(src, ()), "-I", os.path.join(ROOT, "include"), "-I", CSRC,
               "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for src, pr in procs:
        out, _ = pr.communicate()
        out = "\n".join(l for l in out.splitlines() if "not a recognized feature" not in l)
        if pr.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and out.strip():
            print(out)
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH, *objs]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed:\n{res.stdout}")
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
