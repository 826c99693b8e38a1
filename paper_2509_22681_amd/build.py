"""Build libflame_gr.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libflame_gr.so")
MICROBENCH = os.path.join(HERE, "chip_microbench")
SOURCES = ["api.cpp", "plan.cpp", "dso.cpp", "misc.hip", "kernels_f32.hip", "gemm_mfma.hip", "attn_mfma.hip", "k3_mfma.hip", "climber_head.hip"]
# packed fp32 VALU instructions are switched off on purpose: the compiler forms them by itself from plain float
# code and some of their forms have given wrong results on this hardware
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         ]
# keep MFMA accumulators in ordinary VGPRs: the epilogues and the attention SiLU read them with VALU
# instructions, and accumulation registers would need a copy each way
VGPR_FORM = ["-mllvm", "-amdgpu-mfma-vgpr-form"]


def build(verbose: bool = True, jobs: int = 6) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src + ".o")
        objs.append(obj)
        cmd = [hipcc, *FLAGS, *VGPR_FORM, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        while sum(p.poll() is None for _, _, p in procs) >= jobs:
            procs[0][2].wait()
    failed = False
    for src, cmd, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            failed = True
            sys.stderr.write(f"[build] {src} FAILED\n{' '.join(cmd)}\n{out}\n")
        elif verbose and out.strip():
            sys.stderr.write(f"[build] {src}:\n{out}\n")
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = [hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *objs]
    subprocess.run(cmd, check=True)
    if verbose:
        sys.stderr.write(f"[build] wrote {LIB}\n")
    # the box microbenchmarks (a standalone program: profiles/chip_microbench.md is its output)
    subprocess.run([hipcc, *FLAGS, *VGPR_FORM, os.path.join(CSRC, "chip_microbench.hip"), "-o", MICROBENCH], check=True)
    if verbose:
        sys.stderr.write(f"[build] wrote {MICROBENCH}\n")
    return LIB


if __name__ == "__main__":
    build()
