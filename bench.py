#!/usr/bin/env python3
"""Benchmark of the MI355X mLSTM kernels: one "step" = one forward + one backward pass of the
whole hot path (gates, recurrent kernel, parallel kernel, backward recurrence, the three
gradient kernels, gate gradients) over one batch of seeded synthetic input that is already
resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4] [--chunk L] [--variant exp|sig]
                    [--fwd-only] [--no-cpu-baseline] [--no-kernel-events]
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import workloads as wl  # noqa: E402

PEAK_BF16_MFMA = 2.5e15     # FLOP/s, MI355X dense bf16 (no sparsity)
PEAK_FP32_MFMA = 157.3e12   # FLOP/s, MI355X fp32 matrix
PEAK_HBM = 8.0e12           # B/s


def algorithmic_flops(w: wl.Workload, F_causal: float = 0.5):
    """Matmul FLOPs the method itself needs, per kernel family, for the whole workload
    (paper App. F.1 'Numerator', 'Intra Outputs', 'Inter Outputs' rows; App. C.4 for the
    three-product form of each gradient kernel).  Recomputation inside kernels is not counted."""
    tok = w.B * w.NH * w.T            # token-heads
    dd = w.dqk * w.dhv
    intra = F_causal * 2 * w.chunk * (w.dqk + w.dhv)
    fl = {
        "recurrent_fwd": tok * 2 * dd,
        "tile_H": tok * (2 * dd + intra),
        "recurrent_bwd": tok * 2 * dd,
        "tile_dV": tok * (2 * dd + intra),
        "tile_dQ": tok * (2 * dd + intra),
        "tile_dK": tok * (2 * dd + intra),
    }
    fwd = fl["recurrent_fwd"] + fl["tile_H"]
    # fused-minimal backward: S and dS-bar once (2L(d_qk+d_hv)), then dV, dQ, dK (2L(2d_qk+d_hv)),
    # plus dC recurrence, and the three inter-chunk products
    bwd = tok * (8 * dd + F_causal * 2 * w.chunk * (3 * w.dqk + 2 * w.dhv))
    return fl, fwd, bwd


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c4")
    ap.add_argument("--chunk", type=int, default=0)
    ap.add_argument("--variant", default="")
    ap.add_argument("--batch", type=int, default=0)
    ap.add_argument("--fwd-only", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-events", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path shards over batch and heads without "
              "communication; no multi-GPU figure is produced). Run with --gpus 1.", file=sys.stderr)
        return 2

    import torch
    import paper_2503_14376_amd as tfla
    from tests import gpu_util as gu

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    tfla.load_library()   # fails loudly if the HIP library is missing

    w = wl.CONFIGS[args.workload]
    if args.chunk:
        w = dataclasses.replace(w, chunk=args.chunk)
    if args.variant:
        w = dataclasses.replace(w, variant=wl.EXP if args.variant == "exp" else wl.SIG)
    if args.batch:
        w = dataclasses.replace(w, B=args.batch)
    do_bwd = not args.fwd_only
    if do_bwd and not w.backward:
        w = dataclasses.replace(w, backward=True)
    d = wl.make_inputs(w)
    dev = gu.dev_inputs(w, d)
    torch.cuda.synchronize()

    f32 = torch.float32
    B, NH, T = w.B, w.NH, w.T
    ws_f = torch.empty(tfla.workspace_bytes(0, B, NH, T, w.dqk, w.dhv, w.chunk, w.variant, w.dtype), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(max(1, tfla.workspace_bytes(1, B, NH, T, w.dqk, w.dhv, w.chunk, w.variant, w.dtype)) if do_bwd else 1,
                       dtype=torch.uint8, device="cuda")
    fo, bo = {}, {}

    def step():
        tfla.mlstm_fwd(dev["q"], dev["k"], dev["v"], dev["i_pre"], dev["f_pre"], dev.get("C0"), dev.get("n0"),
                       dev.get("m0"), chunk=w.chunk, variant=w.variant, eps=1e-6, workspace=ws_f, out=fo)
        if do_bwd:
            tfla.mlstm_bwd(dev["q"], dev["k"], dev["v"], dev["i_pre"], dev["f_pre"], dev["dH"], fo["n_out"],
                           fo["m_out"], dev.get("C0"), dev.get("n0"), dev.get("m0"), None, chunk=w.chunk,
                           variant=w.variant, eps=1e-6, workspace=ws_b, out=bo)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    use_events = not args.no_kernel_events
    if use_events:
        tfla.profile_enable(16 * (args.steps + 1))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    kernels = {}
    if use_events:
        prof = tfla.profile_read()
        tfla.profile_enable(0)
        kernels = {k_: v_["ms"] / v_["launches"] for k_, v_ in prof.items() if v_["launches"] > 0}

    tokens = w.B * w.T
    value = tokens / (ms_per_step * 1e-3)
    fl, fwd_fl, bwd_fl = algorithmic_flops(w)
    total_fl = fwd_fl + (bwd_fl if do_bwd else 0.0)
    peak = PEAK_BF16_MFMA if w.dtype == wl.BF16 else PEAK_FP32_MFMA

    roof = None
    if kernels:
        cand = {k_: v_ for k_, v_ in kernels.items() if k_ in fl}
        dom = max(cand, key=cand.get)
        ach = fl[dom] / (cand[dom] * 1e-3)
        roof = {"bound": "mfma", "kernel": dom, "achieved": ach / 1e12, "peak": peak / 1e12, "unit": "TFLOP/s",
                "frac": ach / peak, "traffic": None,
                "kernel_ms": {k_: round(v_, 4) for k_, v_ in kernels.items()},
                "kernel_frac": {k_: fl[k_] / (v_ * 1e-3) / peak for k_, v_ in cand.items()}}

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import mlstm_oracle as orc
        nsl = min(4, w.B * w.NH)
        ds = wl.make_inputs(w, heads=nsl)
        oi = gu.oracle_inputs(ds)
        c0 = time.perf_counter()
        orc.recurrent_fwd(**oi, variant=w.variant, eps=1e-6)
        if do_bwd:
            orc.chunkwise_bwd(**oi, dH=gu.flat(ds["dH"]), variant=w.variant, eps=1e-6, chunk=w.chunk)
        c1 = time.perf_counter()
        frac = nsl / float(w.B * w.NH)
        cpu = {"value": tokens * frac / (c1 - c0), "unit": "tokens/s", "cores": int(orc.num_threads()),
               "kind": "oracle", "seconds": c1 - c0,
               "sample": "first %d of %d (batch, head) slices at full T: fp64 step-by-step recurrence forward%s; "
                         "tokens/s scaled by the slice fraction" % (nsl, w.B * w.NH,
                                                                   " + fp64 chunkwise backward (numpy)" if do_bwd else "")}

    line = {
        "metric": "mLSTM fwd+bwd tokens/s" if do_bwd else "mLSTM fwd tokens/s",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == wl.BF16 else "f32", "data": "synthetic",
        "config": {"workload": w.name, "variant": "mLSTMexp" if w.variant == wl.EXP else "mLSTMsig",
                   "B": w.B, "NH": w.NH, "T": w.T, "dqk": w.dqk, "dhv": w.dhv, "chunk": w.chunk,
                   "pass": "fwd+bwd" if do_bwd else "fwd", "states": "element type of q/k/v (bf16), fp32 accumulation"},
        "algorithmic_tflops": total_fl / 1e12,
        "mfma_frac_of_peak_whole_step": total_fl / (ms_per_step * 1e-3) / peak,
        "roofline": roof,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
