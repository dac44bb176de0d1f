"""Builds libqgtc.so (the C-ABI library) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB_DIR = os.path.join(PKG, "lib")
LIB_PATH = os.path.join(LIB_DIR, "libqgtc.so")
OBJ_DIR = os.path.join(PKG, "_build")

SOURCES = ["api.hip", "plan.hip", "pack.hip", "host_pack.hip", "tilemap.hip", "aggregate.hip", "layer.hip", "update.hip", "update_mfma.hip", "probe.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17",
    # no fused multiply-add contraction: the quantizer and the dequantizing
    # epilogue are defined as separately rounded IEEE operations
    "-ffp-contract=off",
    # no compiler-generated packed fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-Wno-inline-asm",   # M0 (lane select of v_writelane) is named as clobbered on purpose
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _run(cmd):
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines()
                    if "packed-fp32-ops" not in l)       # host pass: feature unknown, harmless
    if proc.returncode != 0:
        raise RuntimeError("command failed: " + " ".join(cmd) + "\n" + out)
    return out


def build(verbose: bool = False) -> str:
    """Regenerates the inline-assembly blocks, compiles every source and links
    libqgtc.so.  Always compiles (no up-to-date check)."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    os.makedirs(LIB_DIR, exist_ok=True)
    gen = subprocess.run([sys.executable, os.path.join(CSRC, "gen_popc_blocks.py")],
                         stdout=subprocess.PIPE, check=True, text=True).stdout
    inc = os.path.join(CSRC, "popc_blocks.inc")
    if not os.path.exists(inc) or open(inc).read() != gen:
        with open(inc, "w") as f:
            f.write(gen)
    hipcc = _hipcc()

    def compile_one(src):
        obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
        out = _run([hipcc, *HIPCC_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj])
        if verbose and out.strip():
            print(out)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    # Link against the HIP runtime by soname only (no run path): inside Python the
    # runtime that PyTorch has already loaded must be the one that gets used.
    rocm_lib = os.path.join(os.path.dirname(os.path.dirname(os.path.realpath(hipcc))), "lib")
    _run(["g++", "-shared", "-fPIC", "-o", LIB_PATH, *objs, "-L", rocm_lib, "-lamdhip64"])
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
