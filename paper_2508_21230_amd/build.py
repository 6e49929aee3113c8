"""Builds libejoin.so (the HIP kernels and their C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
SRC = os.path.join(PKG, "csrc", "ejoin.hip")
LIB = os.path.join(PKG, "libejoin.so")
INCLUDE = os.path.join(ROOT, "include")

HIPCC_FLAGS = [
    "-O3",
    "--offload-arch=gfx950",
    # no packed-FP32 VALU instructions: keep the compiler from forming v_pk_*_f32
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-shared", "-fPIC", "-std=c++17",
]


#: ablation builds of the join kernel: name -> extra compiler defines (see the top of csrc/ejoin.hip)
ABLATIONS = {
    "three_stages": ["-DEJOIN_ABL_NSTAGE=3"],
    "no_swizzle": ["-DEJOIN_ABL_NOSWIZZLE"],
    "rowmajor_tiles": ["-DEJOIN_ABL_ROWMAJOR_TILES", "-DEJOIN_ABL_NOALIGN"],
    "no_xcd_align": ["-DEJOIN_ABL_NOALIGN"],
    "no_prefilter": ["-DEJOIN_ABL_NOPREFILTER"],
}
#: measurement builds whose results are meaningless (timing only; see the top of csrc/ejoin.hip and bench_ablation.py --experiments)
EXPERIMENTS = {
    "hot_panels": ["-DEJOIN_EXP_HOT_PANELS"],
    "no_copies": ["-DEJOIN_EXP_NO_COPIES"],
    "cycle_marks": ["-DEJOIN_EXP_CYCLE_MARKS"],
}
ABLATION_DIR = os.path.join(PKG, "ablation")


def _compile(out: str, defines=(), verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        hipcc = "hipcc"
    tmp = out + ".tmp%d" % os.getpid()
    cmd = [hipcc, *HIPCC_FLAGS, *defines, "-I", INCLUDE, "-o", tmp, SRC]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    if verbose:
        print(" ".join(cmd))
    os.replace(tmp, out)
    return out


def build_library(verbose: bool = False) -> str:
    """Compile csrc/ejoin.hip -> libejoin.so (always recompiles; takes a few seconds)."""
    return _compile(LIB, verbose=verbose)


def build_ablations(verbose: bool = False) -> dict:
    """Compile the ablation variants and the two timing-only experiment builds -> ablation/libejoin_<name>.so
    (measurement only, see bench_ablation.py)."""
    os.makedirs(ABLATION_DIR, exist_ok=True)
    return {name: _compile(os.path.join(ABLATION_DIR, f"libejoin_{name}.so"), defs, verbose)
            for name, defs in {**ABLATIONS, **EXPERIMENTS}.items()}


if __name__ == "__main__":
    import sys
    print(build_library(verbose=True))
    if "--ablations" in sys.argv:
        print(build_ablations(verbose=True))
