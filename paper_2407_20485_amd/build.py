"""Builds liba2sf.so (HIP kernels + C ABI) and the stand-alone `ceilings` probe (machine
ceilings the roofline figures are compared with) for gfx950 next to this file.

    python -m paper_2407_20485_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liba2sf.so")
CEILINGS = os.path.join(HERE, "ceilings")
SOURCES = ["a2sf_api.hip", "decode.hip", "select_compact.hip", "prefill_f32.hip", "prefill_bf16.hip",
           "similarity.hip", "chunk.hip"]
# -packed-fp32-ops is switched off: packed fp32 forms have produced wrong results on the
# target machines; the host pass does not know the feature and says so (harmless).
COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Wno-unused-command-line-argument"]
FLAGS = COMMON + ["-fPIC", "-shared"]


def generate() -> None:
    """Writes the generated instruction stream(s) the kernels include."""
    subprocess.run([sys.executable, os.path.join(CSRC, "gen_attn_fwd128x2.py")], check=True,
                   capture_output=True)


def _hipcc(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}):\n{err}")
    if verbose and err.strip():
        print(err, file=sys.stderr)


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    generate()
    _hipcc([hipcc, *FLAGS, *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB], verbose)
    _hipcc([hipcc, *COMMON, os.path.join(CSRC, "ceilings.hip"), "-o", CEILINGS], verbose)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
