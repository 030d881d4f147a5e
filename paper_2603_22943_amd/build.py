"""Build libtaq.so (gfx950 only) in-tree with hipcc.

    python -m paper_2603_22943_amd.build

Flags that matter for parity with the float32-defined quantizers:
  -ffp-contract=off                          no silent FMA contraction (FMAs are explicit where wanted)
  -fhip-fp32-correctly-rounded-divide-sqrt   IEEE float32 division
  -fno-honor-nans                            inputs are finite by contract; saves the NaN-quieting
                                             instruction in front of every max (infinities stay honoured:
                                             the -inf token bias relies on them)
and packed-fp32 instructions are switched off for the device pass.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtaq.so")
SOURCES = ["taq_fused_d40.hip", "taq_fused_d80.hip", "taq_fused_d64.hip", "taq_fused_mid160.hip", "taq_fused_mid64.hip",
           "taq_fused.hip", "taq_api.hip", "taq_quant.hip", "taq_gemm.hip", "taq_attn.hip", "taq_fp.hip"]


def hipcc_path() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found: libtaq needs the ROCm toolchain")


def build_lib(verbose: bool = True) -> str:
    """Compile every source to an object (in parallel: one hipcc per file) and link libtaq.so."""
    from concurrent.futures import ThreadPoolExecutor

    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    flags = [
        "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
        "-ffp-contract=off", "-fhip-fp32-correctly-rounded-divide-sqrt", "-fno-honor-nans",
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-Wall", "-Wno-unused-function",
        "-I", os.path.join(os.path.dirname(HERE), "include"),
    ] + os.environ.get("TAQ_EXTRA_HIPCC_FLAGS", "").split()
    hipcc = hipcc_path()

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
        if verbose and out.strip():
            print(out, flush=True)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + out)

    objs = [os.path.join(objdir, s.replace(".hip", ".o")) for s in SOURCES]
    jobs = [[hipcc] + flags + ["-c", os.path.join(CSRC, s), "-o", o] for s, o in zip(SOURCES, objs)]
    with ThreadPoolExecutor(max_workers=min(len(jobs), os.cpu_count() or 1)) as pool:
        list(pool.map(run, jobs))
    run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs)
    return LIB


if __name__ == "__main__":
    build_lib()
    print("built", LIB)
    sys.exit(0)
