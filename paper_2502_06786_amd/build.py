"""Build libmq.so (the C-ABI library of include/mq.h) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmq.so")
# measurement-only kernels used by bench.py (matrix-core and read ceilings): a library of their own
PROBE_DIR = os.path.join(HERE, "bench_probes")
PROBE_LIB = os.path.join(PROBE_DIR, "libmq_probe.so")
SOURCES = ["mq_quantize.hip", "mq_slice.hip", "mq_gemv.hip", "mq_gemv_quad.hip", "mq_gemv_ovf.hip", "mq_gemv_reg.hip", "mq_linear.hip", "mq_ffn.hip", "mq_loss.hip", "mq_clip.hip", "mq_affine.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
    # packed fp32 instructions are kept out of every kernel
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def build(verbose: bool = False) -> str:
    """Compile every HIP source, link libmq.so and the bench-only libmq_probe.so; returns the path of libmq.so."""
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        cmd = ["hipcc", *HIPCC_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    cmd = ["hipcc", *HIPCC_FLAGS, "-shared", os.path.join(PROBE_DIR, "probes.hip"), "-o", PROBE_LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    procs.append(("probes.hip", subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        # hipcc's host pass warns that it does not know the packed-fp32 feature: harmless
        out = "\n".join(ln for ln in out.splitlines() if "packed-fp32-ops" not in ln)
        if out.strip():
            print(out, file=sys.stderr)
        if p.returncode != 0:
            failed = True
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
