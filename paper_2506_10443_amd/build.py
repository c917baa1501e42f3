"""Builds libmnnq.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB_DIR = os.path.join(HERE, "lib")
LIB = os.path.join(LIB_DIR, "libmnnq.so")

SOURCES = ["mnnq_api.hip", "mnnq_pack.hip", "mnnq_quant_act.hip", "mnnq_decode.hip",
           "mnnq_prefill.hip", "mnnq_prefill6.hip", "mnnq_prefill_f16.hip", "mnnq_f16.hip", "mnnq_skinny.hip"]
# measurement helpers of bench.py: a library of their own, not part of the product's C-ABI
BENCH_SOURCES = ["bench_kernels.hip"]
BENCH_LIB = os.path.join(LIB_DIR, "libmnnq_bench.so")
# The quantizers are fixed sequences of IEEE binary32 operations: no contraction.
STRICT_FP = {"mnnq_pack.hip", "mnnq_quant_act.hip", "mnnq_decode.hip"}
# MFMA results stay in architectural VGPRs so that the VALU epilogue reads them directly.
MFMA_VGPR = {"mnnq_prefill.hip", "mnnq_prefill6.hip", "mnnq_prefill6.hip", "mnnq_prefill_f16.hip", "mnnq_skinny.hip", "bench_kernels.hip"}

COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
          "-fhip-fp32-correctly-rounded-divide-sqrt",
          # packed fp32 VALU forms are kept out of the generated code
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Wall", "-Wno-unused-function"]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    cmd = [hipcc()] + COMMON + (["-ffp-contract=off"] if src in STRICT_FP else []) + \
        (["-mllvm", "-amdgpu-mfma-vgpr-form"] if src in MFMA_VGPR else []) + \
        ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, r.stdout, r.stderr))
    # the host pass warns that it does not know the packed-fp32 feature; drop that line
    msgs = [l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip()]
    if msgs:
        sys.stderr.write("\n".join(msgs) + "\n")
    return obj


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    os.makedirs(LIB_DIR, exist_ok=True)
    with ThreadPoolExecutor(8) as pool:
        objs = list(pool.map(_compile, SOURCES + BENCH_SOURCES))
    for lib, lib_objs in ((LIB, objs[:len(SOURCES)]), (BENCH_LIB, objs[len(SOURCES):])):
        tmp = lib + ".tmp.%d" % os.getpid()
        cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + lib_objs
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n%s\n%s" % (r.stdout, r.stderr))
        os.replace(tmp, lib)
        if verbose:
            print("built", lib)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
