"""Builds liblrnnx.so (the C-ABI scan library) for gfx950 with hipcc, in-tree.

    python -m paper_2602_08810_amd.build

Each .hip file under csrc/ is compiled to an object in parallel, then linked into
paper_2602_08810_amd/liblrnnx.so; csrc/valu_probe.hip becomes the stand-alone program
paper_2602_08810_amd/valu_probe.  hipcc cross-compiles: no GPU is needed to build.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "liblrnnx.so")
PROBE = os.path.join(HERE, "valu_probe")
SOURCES = ["api.hip", "selective_fwd.hip", "selective_bwd.hip", "selective_bwd_carry.hip", "selective_cplx_fwd.hip", "selective_cplx_bwd.hip", "lti_scan.hip", "diag_scan.hip", "step.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-munsafe-fp-atomics",
    # packed fp32 VALU forms are switched off for the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{r.stderr}")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr}")
    if verbose:
        print(f"built {LIB}")
    # the stand-alone issue-rate probe of the vector ALU (bench.py --alu-probe runs it)
    r = subprocess.run([HIPCC, *FLAGS, os.path.join(CSRC, "valu_probe.hip"), "-o", PROBE], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on valu_probe.hip:\n{r.stderr}")
    if verbose:
        print(f"built {PROBE}")
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
