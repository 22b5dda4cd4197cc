"""Build libcitrus.so (HIP, gfx950) in-tree with hipcc.

Usage: python -m paper_2406_12018_amd.build
"""

from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libcitrus.so")
SOURCES = ["citrus_api.hip", "attn_generic.hip", "attn_mfma.hip", "instr_strip.hip", "decode_attn.hip", "rope.hip", "select_compact.hip", "probe.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # keep MFMA accumulators in VGPRs: the softmax rescale touches them with vector ALU ops, and
    # AGPR-resident accumulators cost a copy per register and per loop iteration
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",
    "-Wall", "-Wno-unused-function",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


# The attention kernel fixes the issue order of its MFMAs and exponentials with volatile asm statements, which
# hides those instructions from the compiler's hazard recogniser: no compiler-visible instruction may read an
# accumulator sooner than the MFMA that writes it completes, and the kernel keeps a full MFMA group (or explicit
# wait states) in between.  Whether the register allocator respects that was checked, with the parity and the
# run-twice bit-identity tests on an MI355X, for the compiler below.  Another compiler is not refused, but the
# build says so loudly: re-run `pytest -m gpu` (test_gpu_parity.py, test_gpu_random_shapes.py) before trusting it.
VALIDATED_COMPILER = "AMD clang version 22.0.0git (https://github.com/RadeonOpenCompute/llvm-project roc-7.2.0 26014"


def compiler_version(exe: str) -> str:
    res = subprocess.run([exe, "--version"], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    lines = [l.strip() for l in res.stdout.splitlines() if "clang version" in l]
    return lines[0] if lines else res.stdout.strip().splitlines()[0] if res.stdout.strip() else "unknown"


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: cannot build libcitrus.so")
    return exe


def build(verbose: bool = True) -> str:
    exe = hipcc()
    version = compiler_version(exe)
    if verbose:
        print(f"compiler: {version}", flush=True)
    if not version.startswith(VALIDATED_COMPILER):
        print("WARNING: libcitrus.so is being built with a compiler other than the one its hand-ordered MFMA "
              f"pipeline was validated with ({VALIDATED_COMPILER} ...): run the GPU parity and bit-identity tests "
              "before use", file=sys.stderr, flush=True)
    cmd = [exe] + HIPCC_FLAGS + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if verbose and out.strip():
        print(out, flush=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    return LIB_PATH


if __name__ == "__main__":
    build()
    sys.exit(0)
