"""Build ``libbuzz.so`` (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libbuzz.so")
# (source, object stem, extra defines); the attention kernels are one translation unit per dtype
SOURCES = [("buzz_api.cpp", "buzz_api", []), ("evict_kernels.hip", "evict_kernels", []),
           # matrix-core results go to ordinary registers: the scoring kernels read every one of them with
           # vector instructions, and a copy out of the accumulation registers per element costs 15% of them
           ("prefill_kernels.hip", "prefill_kernels", ["-mllvm", "-amdgpu-mfma-vgpr-form"]),
           ("attn_kernels.hip", "attn_fp32", ["-DBUZZ_TU=0"]), ("attn_kernels.hip", "attn_fp16", ["-DBUZZ_TU=1"]),
           ("attn_kernels.hip", "attn_bf16", ["-DBUZZ_TU=2"]), ("attn_kernels.hip", "attn_common", ["-DBUZZ_TU=3"])]
FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-fno-gpu-rdc",
    # packed fp32 VALU forms are switched off for the whole library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def build(verbose: bool = False) -> str:
    """Compile every source and link the shared library; always recompiles."""
    objs = []
    procs = []
    for src, stem, defs in SOURCES:
        obj = os.path.join(CSRC, stem + ".o")
        cmd = ["hipcc", "-x", "hip", *FLAGS, *defs, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
               "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        # the host pass does not know the packed-fp32 feature name; that warning is expected
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if out.strip() and (verbose or p.returncode):
            print(out, file=sys.stderr)
        failed |= p.returncode != 0
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
