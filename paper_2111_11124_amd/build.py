"""Build libmesa.so in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

PKG = Path(__file__).resolve().parent
CSRC = PKG / "csrc"
INCLUDE = PKG.parent / "include"
LIB = PKG / "libmesa.so"
OBJ = PKG / "_build"
SOURCES = ["stream_kernels.hip", "softmax_fwd.hip", "softmax_bwd.hip", "layernorm_fwd.hip", "layernorm_bwd.hip", "linear_dw.hip", "attn_matmul_bwd.hip", "lowbit.hip", "conv_dw.hip", "mfma_probe.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# -ffp-contract=off: no implicit fused multiply-adds anywhere; kernels that may fuse call fmaf.
# The packed-fp32 feature is switched off as this pool requires.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden", "-ffp-contract=off",
         "-fhip-fp32-correctly-rounded-divide-sqrt", "-fno-gpu-flush-denormals-to-zero",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
         f"-I{INCLUDE}", f"-I{CSRC}"]


def _compile(src: str) -> Path:
    OBJ.mkdir(exist_ok=True)
    out = OBJ / (src + ".o")
    cmd = [HIPCC, *FLAGS, "-c", str(CSRC / src), "-o", str(out)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError(f"hipcc failed on {src}")
    errs = [l for l in r.stderr.splitlines() if "warning" in l and "packed-fp32-ops" not in l and "unused-value" not in l]
    if errs:
        sys.stderr.write("\n".join(errs[:20]) + "\n")
    return out


def build(verbose: bool = True) -> Path:
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(_compile, SOURCES))
    tmp = LIB.with_suffix(f".tmp{os.getpid()}.so")
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(tmp), *map(str, objs)]
    subprocess.run(cmd, check=True)
    os.replace(tmp, LIB)
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build()
