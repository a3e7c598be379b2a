"""Build the HIP library in-tree: paper_2510_15964_amd/liblx_sparse.so (gfx950)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblx_sparse.so")
SOURCES = ["lx_api.hip", "compact.hip", "ffn_f32.hip", "ffn_bf16.hip", "predict_bf16.hip", "lora_bf16.hip",
           "attn_bf16.hip", "attn_f32.hip", "probe.hip"]
# -Wno-inline-asm: the DMA helpers name m0 (a register the compiler reserves) as clobbered, which
# is the point, and clang warns about every such statement
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-inline-asm",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *FLAGS, "-shared", "-Wl,--no-undefined", *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB]
    if verbose:
        cmd.insert(1, "-Rpass-analysis=kernel-resource-usage")
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines()
                    if "not a recognized feature" not in l)
    if r.returncode != 0:
        if os.path.exists(LIB):
            os.remove(LIB)          # never leave a stale library behind a failed build
        raise RuntimeError("hipcc failed:\n" + err)
    if err.strip():
        sys.stderr.write(err + "\n")
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
