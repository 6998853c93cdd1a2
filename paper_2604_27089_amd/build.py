"""Build the C-ABI library: hipcc, gfx950 only, in-tree.

    python -m paper_2604_27089_amd.build

produces paper_2604_27089_amd/libsp_hotpath.so next to this file.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libsp_hotpath.so")
# The same sources with every hand-scheduled MFMA padded by full waits and wait states (-DSP_PADDED_MFMA):
# slow, hazard-proof, bit-identical by construction; a GPU test compares the two builds.
LIB_PADDED = os.path.join(HERE, "libsp_hotpath_padded.so")
SOURCES = ["sp_api.hip", "relayout.hip", "doc_bounds.hip", "attn_fwd.hip", "attn_bwd.hip", "attn_bwd_dkdv.hip", "attn_bwd_dq.hip", "attn_merge.hip", "pointwise.hip"]
FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-Wall", "-Wextra",
         "-Wno-unused-command-line-argument", "-Wno-unused-parameter",
         # keep the compiler from forming packed-fp32 VALU instructions
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(job) -> str:
    src, padded = job
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + (".padded.o" if padded else ".o"))
    cmd = ["hipcc", *FLAGS, *(["-DSP_PADDED_MFMA"] if padded else []), "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines()
                    if "packed-fp32-ops' is not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(jobs: int = 6) -> str:
    os.makedirs(OBJ, exist_ok=True)
    work = [(s, False) for s in SOURCES] + [(s, True) for s in SOURCES]
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, work))
    n = len(SOURCES)
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs[:n], "-o", LIB], check=True)
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs[n:], "-o", LIB_PADDED], check=True)
    return LIB


if __name__ == "__main__":
    print(build())
