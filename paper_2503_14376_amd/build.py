"""Builds libtfla_mlstm.so (HIP, gfx950) in-tree with hipcc.  Usage: python -m paper_2503_14376_amd.build"""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "lib", "libtfla_mlstm.so")

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-Wno-inline-asm", "-Wno-pass-failed"]

# (source, object name, extra defines)
# recurrent.hip: MFMA accumulators in ordinary VGPRs (the kernel also scales and stores them with
# vector ALU instructions, which cannot read accumulation registers)
UNITS = [("api.hip", "api.o", []), ("gates.hip", "gates.o", []), ("step.hip", "step.o", []), ("norm.hip", "norm.o", []), ("pad.hip", "pad.o", []),
         ("recurrent.hip", "recurrent.o", ["-mllvm", "-amdgpu-mfma-vgpr-form"])] + [
    # tile kernels: the start-up loop over X and state slices must unroll completely (its items differ in kind and
    # index registers by compile-time constants); with the widest shapes its body exceeds the default size limit
    # (accumulators in ordinary VGPRs as for recurrent.hip: the dK kernel then needs no accumulation registers at all)
    ("tile_inst.hip", "tile_mode%d.o" % m, ["-DTFLA_TILE_MODE=%d" % m, "-mllvm", "-pragma-unroll-threshold=200000",
                                            "-mllvm", "-amdgpu-mfma-vgpr-form"]) for m in range(4)]


def _compile(unit):
    src, obj, defs = unit
    cmd = ["hipcc", *FLAGS, *defs, "-c", os.path.join(CSRC, src), "-o", os.path.join(OBJ, obj)]
    p = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in p.stderr.splitlines() if "packed-fp32-ops" not in l)
    return unit, p.returncode, err


def build(verbose: bool = True, jobs: int = 8) -> str:
    os.makedirs(OBJ, exist_ok=True)
    os.makedirs(os.path.dirname(LIB), exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as ex:
        results = list(ex.map(_compile, UNITS))
    for unit, rc, err in results:
        if err.strip() and verbose:
            print(err, file=sys.stderr)
        if rc != 0:
            raise RuntimeError("hipcc failed for %s" % unit[0])
    objs = [os.path.join(OBJ, u[1]) for u in UNITS]
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build())
