"""Builds libtom_oqm.so (gfx950 kernels + C ABI) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libtom_oqm.so")
OBJ = os.path.join(HERE, "_build")
SELFCHECK = os.path.join(HERE, "selfcheck_division.bin")

SOURCES = ["oqm_api.hip", "oqm_quantize.hip", "oqm_quantize_tokens.hip", "oqm_dequant.hip", "oqm_score.hip",
           "oqm_topk.hip"]
# benchmark-only helpers (stream probes, timing events): a shared object of their own that only
# bench.py loads; nothing of it is in the library or in its ABI header
BENCH_LIB = os.path.join(HERE, "libtom_bench_probe.so")

# -ffp-contract=off: the codes, scale/zero and dequantized values must be single, separately
# rounded IEEE operations.  -fno-honor-nans (inputs are finite by contract) only lets min/max
# compile to one instruction each; it changes no result on finite data.
COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
          "-fno-honor-nans", "-fvisibility=hidden", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Wall", "-Wno-unused-result", "-I", INCLUDE, "-I", CSRC]


# Per-file additions.  The score contraction keeps its float64 accumulators in ordinary vector
# registers: without this the compiler moves all 32 of them to the accumulation file and back
# around every staged chunk (64 copies per 32 MFMAs).
EXTRA = {"oqm_score.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)

    def compile_one(src: str) -> str:
        obj = os.path.join(OBJ, src.replace(".hip", ".o"))
        cmd = ["hipcc", *COMMON, *EXTRA.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}\n{r.stderr}")
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    cmd = ["hipcc", *COMMON, "-shared", os.path.join(CSRC, "bench_probe.hip"), "-o", BENCH_LIB]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"bench probe build failed:\n{r.stdout}\n{r.stderr}")
    # stand-alone GPU program that checks the kernels' division shortcuts exhaustively
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-ffp-contract=off",
           "-Wno-unused-result", "-I", INCLUDE, "-I", CSRC,
           os.path.join(CSRC, "selfcheck_division.hip"), "-o", SELFCHECK]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"selfcheck build failed:\n{r.stdout}\n{r.stderr}")
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
