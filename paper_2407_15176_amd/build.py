"""Builds libreattn.so (hand-written HIP, gfx950 only) in-tree with hipcc.

Every source is compiled to an object of its own (in parallel) and the objects are linked
into the shared library.  `build_library(force=True)` recompiles everything; without
`force` only sources newer than their object (or older than a shared header) are rebuilt.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libreattn.so")
SOURCES = ["api.hip", "score_scan.hip", "score_gemm.hip", "prefill_select.hip", "topk.hip", "decode_select.hip", "rope.hip",
           "attend.hip", "attend_prefill.hip", "vote.hip", "vote_scan.hip", "vote_gemm.hip", "attend_shared.hip"]
HEADERS = [os.path.join(CSRC, "common.hpp"), os.path.join(CSRC, "select.hpp"), os.path.join(CSRC, "vote_scan.hpp"), os.path.join(HERE, "..", "include", "reattn.h")]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]
# vote_gemm.hip runs one wave per SIMD with more than 256 registers: there the compiler would put every
# matrix result into the accumulation half of the register file and copy it out for the vector unit.
FILE_FLAGS = {"vote_gemm.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


def _stale(src: str, obj: str) -> bool:
    if not os.path.exists(obj):
        return True
    t = os.path.getmtime(obj)
    return any(os.path.getmtime(f) > t for f in [src, *HEADERS] if os.path.exists(f))


def _compile(src: str, obj: str, verbose: bool) -> None:
    cmd = [HIPCC, *FLAGS, *FILE_FLAGS.get(os.path.basename(src), []), "-c", "-o", obj, src]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass does not know the packed-fp32 target feature and says so: harmless
    noise = "is not a recognized feature for this target"
    text = "\n".join(l for l in r.stdout.splitlines() if noise not in l)
    if text.strip():
        print(text, flush=True)
    if r.returncode:
        raise RuntimeError(f"hipcc failed on {src}")


def build_library(verbose: bool = False, force: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    jobs = []
    for s in SOURCES:
        src, obj = os.path.join(CSRC, s), os.path.join(OBJ, s.replace(".hip", ".o"))
        if force or _stale(src, obj):
            jobs.append((src, obj))
    with ThreadPoolExecutor(max_workers=min(8, max(1, len(jobs)))) as ex:
        for f in [ex.submit(_compile, src, obj, verbose) for src, obj in jobs]:
            f.result()
    objs = [os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES]
    if jobs or not os.path.exists(LIB):
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose="-v" in sys.argv, force="--force" in sys.argv))
