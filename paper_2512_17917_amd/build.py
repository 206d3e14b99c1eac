"""Compile the HIP sources in csrc/ into paper_2512_17917_amd/libkvr.so for gfx950.

hipcc cross-compiles without a GPU.  Objects go to paper_2512_17917_amd/_build/.
Usage: python -m paper_2512_17917_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libkvr.so")
OBJ_DIR = os.path.join(HERE, "_build")

SOURCES = ["kvr_api.hip", "kvr_reconstruct.hip", "kvr_attend.hip", "kvr_attend_staged.hip", "kvr_attend_staged64.hip", "kvr_attend_staged_r4.hip", "kvr_attend_retained.hip", "kvr_select.hip",
           "kvr_encode.hip", "kvr_swap.hip", "kvr_attend_multi.hip", "kvr_attend_multi_staged.hip"]

# packed-FP32 instruction selection is switched off on purpose (ordinary float
# code only); the host pass warns that it does not know the feature.
HIP_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wno-unused-command-line-argument"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(" ".join(cmd) + "\n" + r.stdout + r.stderr)
        raise RuntimeError("hipcc failed: " + cmd[-1])
    return r


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    hipcc = _hipcc()
    jobs = []
    for s in SOURCES:
        obj = os.path.join(OBJ_DIR, s.replace(".hip", ".o"))
        jobs.append((obj, [hipcc, *HIP_FLAGS, "-c", os.path.join(CSRC, s), "-o", obj]))
    with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as ex:
        for r in ex.map(lambda j: _run(j[1]), jobs):
            if verbose and r.stderr:
                sys.stderr.write(r.stderr)
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", OUT, *[j[0] for j in jobs]])
    return OUT


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
