"""Build ``libsablock.so`` (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""

from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libsablock.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

SOURCES = ["api.hip", "score_generic.hip", "score_mfma.hip", "refine.hip", "search_select.hip", "compact.hip", "segment.hip", "decode.hip", "window_attn.hip"]
FLAGS = ["-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden", "--offload-arch=gfx950", "-Wall", "-Wno-unused-function",
         # keep packed fp32 instructions out of the generated code
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # MFMA results and C operands in ordinary VGPRs (A/B operands may still sit in accumulation registers)
         "-mllvm", "-amdgpu-mfma-vgpr-form=1"]


def _compile(src: str, force: bool) -> str:
    s = os.path.join(CSRC, src)
    o = os.path.join(OBJ, src.replace(".hip", ".o"))
    deps = [s, os.path.join(CSRC, "sablock_internal.h"), os.path.join(HERE, "..", "include", "sablock.h")]
    if force or not os.path.exists(o) or os.path.getmtime(o) < max(os.path.getmtime(d) for d in deps):
        subprocess.run([HIPCC, *FLAGS, "-c", s, "-o", o], check=True)
    return o


def build(force: bool = True, jobs: int = 6) -> str:
    """Compile every source and link the shared library; returns its path."""
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), SOURCES))
    subprocess.run([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *objs], check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv))
