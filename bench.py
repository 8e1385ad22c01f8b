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
DEFAULT_CHUNK = 256          # chunk size of the headline workload (c4)


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


def algorithmic_bytes(w: wl.Workload, es: int):
    """HBM bytes each kernel must move per launch if every operand is read once and every result
    written once: the sequence operands, one set of chunk states (stored in the element type of
    q/k/v), the output block.  Gate vectors (a few fp32 per token) are included."""
    tok = w.B * w.NH * w.T
    st = w.B * w.NH * (w.T // w.chunk) * w.dqk * w.dhv * es
    g = tok * 4
    rec = tok * (w.dqk + w.dhv) * es + st + 2 * g
    if es == 2:
        # fp32 copies of the state at the block boundaries of the anchored forget-gate gradient scan (every fourth
        # chunk, blocks of at most 2048 steps): the forward launch writes them, the reversed launch reads them
        nc = w.T // w.chunk
        G = 2 if max(w.dqk, w.dhv) > 512 else (4 if 4 * w.chunk <= 2048 else max(1, 2048 // w.chunk))
        rec += w.B * w.NH * max(0, (nc + G - 1) // G - 1) * w.dqk * w.dhv * 4
    # the weighted intra-chunk matrix E, lower triangle: where the contraction over d_hv is wider than 256 columns
    # (bf16 path) dQ writes it and dK reads it instead of dH; narrower heads recompute it in dK
    shares_e = es == 2 and w.dhv > 256
    etri = tok * w.chunk * es // 2 if shares_e else 0
    dk_in = etri if shares_e else tok * w.dhv * es
    return {
        "recurrent_fwd": rec,
        "recurrent_bwd": rec,
        "tile_H": tok * (2 * w.dqk + w.dhv) * es + st + tok * w.dhv * es + 4 * g,
        "tile_dV": tok * (2 * w.dqk + w.dhv) * es + st + tok * w.dhv * es + 3 * g,
        "tile_dQ": tok * (2 * w.dhv + 2 * w.dqk) * es + st + tok * w.dqk * es + etri + 4 * g,
        "tile_dK": tok * (w.dhv + 2 * w.dqk) * es + st + tok * w.dqk * es + dk_in + 4 * g,
    }


def profiled_traffic():
    """HBM bytes per launch (fetched + written) of each kernel at the default workload (c4, chunk 256,
    exponential gate), read from the committed summary of the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
    script (profiles/hbm_traffic_c4.txt, column total_MB; the counters are scaled there by what they read for a
    1 GiB copy kernel).  A figure from that profile, not a measurement of the present run: the bench line labels it
    so.  Returns {} when the file is absent."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_c4.txt")
    modes = {"0": "tile_kernel<H>", "1": "tile_kernel<dV>", "2": "tile_kernel<dQ>", "3": "tile_kernel<dK>"}
    out = {}
    try:
        for line in open(path):
            f = line.split()
            try:
                total = float(f[-1]) * 1e6
            except (IndexError, ValueError):
                continue
            if line.startswith("recurrent_kernel_bf16"):
                out["recurrent_kernel"] = total
            elif line.startswith("tile_kernel_bf16<"):
                # template arguments <D1, BD2, NW, MODE, ...>
                targs = line[line.index("<") + 1:line.index(">")].replace(" ", "").split(",")
                if len(targs) >= 4 and targs[3] in modes:
                    out[modes[targs[3]]] = total
    except OSError:
        pass
    return out


def step_bench(args) -> int:
    """Generation: one recurrent step (tfla_mlstm_step) per launch at the 7B head shape, state resident in
    HBM and updated in place.  A secondary line (`--workload step`); the default line is the training step."""
    import torch
    import paper_2503_14376_amd as tfla
    tfla.load_library()
    B, NH, dqk, dhv = (args.batch or 8), 8, 256, 512
    variant = wl.SIG if args.variant == "sig" else wl.EXP
    g = torch.Generator(device="cuda").manual_seed(1005)
    bf = torch.bfloat16
    q = torch.randn((B, NH, dqk), device="cuda", generator=g).to(bf)
    k = torch.randn((B, NH, dqk), device="cuda", generator=g).to(bf)
    v = torch.randn((B, NH, dhv), device="cuda", generator=g).to(bf)
    ip = torch.randn((B, NH), device="cuda", generator=g)
    fp = torch.randn((B, NH), device="cuda", generator=g) + 3.0
    C = 0.1 * torch.randn((B, NH, dqk, dhv), device="cuda", generator=g)
    n = [0.1 * torch.randn((B, NH, dqk), device="cuda", generator=g), torch.empty((B, NH, dqk), device="cuda")]
    m = [torch.zeros((B, NH), device="cuda"), torch.empty((B, NH), device="cuda")]
    h = torch.empty((B, NH, dhv), device="cuda", dtype=bf)
    outs = [{"h": h, "C": C, "n": n[1], "m": m[1]}, {"h": h, "C": C, "n": n[0], "m": m[0]}]
    it = [0]

    def step():
        i = it[0] & 1
        tfla.mlstm_step(q, k, v, ip, fp, C, n[i], m[i], variant=variant, eps=1e-6, out=outs[i])
        it[0] += 1

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    tfla.profile_enable(2 * (args.steps + 1))
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    prof = tfla.profile_read()
    tfla.profile_enable(0)
    kms = prof["recurrent_step"]["ms"] / max(1, prof["recurrent_step"]["launches"])
    # per step and head (App. F.2, memory operations of the recurrent formulation, fp32 states and gates)
    per_head = 2 * 4 + 2 * (dhv + dqk) * 2 + 2 * (dhv * dqk + (dqk + 1 if variant == wl.EXP else 0)) * 4
    byts = per_head * B * NH
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import mlstm_oracle as orc
        T = 256
        f64 = lambda t: t.float().cpu().numpy().astype(np.float64)
        rep = lambda t: np.repeat(f64(t).reshape((B * NH, 1) + tuple(t.shape[2:])), T, axis=1)
        c0 = time.perf_counter()
        orc.recurrent_fwd(rep(q), rep(k), rep(v), np.repeat(f64(ip).reshape(B * NH, 1), T, axis=1),
                          np.repeat(f64(fp).reshape(B * NH, 1), T, axis=1), f64(C).reshape(B * NH, dqk, dhv),
                          f64(n[0]).reshape(B * NH, dqk), f64(m[0]).reshape(B * NH), variant=variant, eps=1e-6)
        c1 = time.perf_counter()
        cpu = {"value": B * T / (c1 - c0), "unit": "tokens/s", "cores": int(orc.num_threads()), "kind": "oracle",
               "seconds": c1 - c0, "sample": "%d steps of the fp64 step-by-step recurrence for all %d heads" % (T, B * NH)}
    line = {"metric": "mLSTM recurrent step (generation) tokens/s at NH=8, dqk=256, dhv=512", "value": B / (ms * 1e-3),
            "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "step", "variant": "mLSTMexp" if variant == wl.EXP else "mLSTMsig", "B": B, "NH": NH,
                       "dqk": dqk, "dhv": dhv, "state": "fp32, updated in place"},
            "roofline": {"bound": "hbm", "kernel": "step_kernel", "achieved": byts / (kms * 1e-3) / 1e9,
                         "peak": PEAK_HBM / 1e9, "unit": "GB/s", "frac": byts / (kms * 1e-3) / PEAK_HBM, "traffic": None,
                         "avg_launch_ms": kms, "algorithmic_bytes_per_launch": byts},
            "cpu_baseline": cpu}
    print(json.dumps(line))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="c4")
    ap.add_argument("--chunk", type=int, default=0)
    ap.add_argument("--variant", default="")
    ap.add_argument("--batch", type=int, default=0)
    ap.add_argument("--seq-len", type=int, default=0, help="override T of the workload (a secondary line)")
    ap.add_argument("--head-dim", type=int, default=0,
                    help="head-dimension sweep point of App. E.3: dqk = dhv = this value, NH = 4096 / value, B = 4 "
                         "(unless --batch), T = 8192; a secondary line")
    ap.add_argument("--tile-width", type=int, default=0,
                    help="tile-size sweep: output-column block of the tiled kernels (64 or 128; 0 = the library's choice)")
    ap.add_argument("--fwd-only", action="store_true")
    ap.add_argument("--recompute", action="store_true",
                    help="do not hand the forward workspace to the backward call (gates and chunk states are recomputed)")
    ap.add_argument("--layer", action="store_true",
                    help="time the layer entry points (gate soft-cap 15, cell, LayerNorm, output gate) instead of the "
                         "cell alone; a secondary line, the default line is the cell")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-events", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="replay one captured HIP graph of the step instead of launching every step eagerly "
                         "(measured slightly slower than eager launches on this stack)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch one plain 1 GiB device copy kernel (the known-size reference that the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run are scaled by)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path shards over batch and heads without "
              "communication; no multi-GPU figure is produced). Run with --gpus 1.", file=sys.stderr)
        return 2

    import torch
    import paper_2503_14376_amd as tfla

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    tfla.load_library()   # fails loudly if the HIP library is missing
    if args.tile_width:
        tfla.tile_width(args.tile_width)
    if args.workload == "step":
        return step_bench(args)

    w = wl.CONFIGS[args.workload]
    if args.chunk:
        w = dataclasses.replace(w, chunk=args.chunk)
    if args.variant:
        w = dataclasses.replace(w, variant=wl.EXP if args.variant == "exp" else wl.SIG)
    if args.head_dim:
        w = dataclasses.replace(w, name="headdim%d" % args.head_dim, dqk=args.head_dim, dhv=args.head_dim,
                                NH=4096 // args.head_dim, B=4, T=8192)
    if args.batch:
        w = dataclasses.replace(w, B=args.batch)
    if args.seq_len:
        w = dataclasses.replace(w, T=args.seq_len)
    do_bwd = not args.fwd_only
    if do_bwd and not w.backward:
        w = dataclasses.replace(w, backward=True)
    d = wl.make_layer_inputs(w) if args.layer else wl.make_inputs(w)
    dev = {key: wl.to_dev(val, w.dtype if key in ("q", "k", "v", "dH", "o_pre") else wl.F32) for key, val in d.items()}
    torch.cuda.synchronize()

    f32 = torch.float32
    B, NH, T = w.B, w.NH, w.T
    wsb = tfla.layer_workspace_bytes if args.layer else tfla.workspace_bytes
    ws_f = torch.empty(wsb(0, B, NH, T, w.dqk, w.dhv, w.chunk, w.variant, w.dtype), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(max(1, wsb(1, B, NH, T, w.dqk, w.dhv, w.chunk, w.variant, w.dtype)) if do_bwd else 1,
                       dtype=torch.uint8, device="cuda")
    fo, bo = {}, {}

    lkw = dict(chunk=w.chunk, variant=w.variant, eps=1e-6, gate_softcap=15.0, norm_kind=tfla.NORM_LAYER, norm_eps=1e-6)

    def layer_step():
        tfla.mlstm_layer_fwd(dev["q"], dev["k"], dev["v"], dev["i_pre"], dev["f_pre"], dev["o_pre"], dev["gamma"],
                             dev["beta"], workspace=ws_f, out=fo, **lkw)
        if do_bwd:
            tfla.mlstm_layer_bwd(dev["q"], dev["k"], dev["v"], dev["i_pre"], dev["f_pre"], fo["H"], dev["dH"],
                                 dev["o_pre"], dev["gamma"], dev["beta"], fo["n_out"], fo["m_out"], workspace=ws_b,
                                 out=bo, fwd_workspace=None if args.recompute else ws_f, **lkw)

    def step():
        if args.layer:
            return layer_step()
        tfla.mlstm_fwd(dev["q"], dev["k"], dev["v"], dev["i_pre"], dev["f_pre"], dev.get("C0"), dev.get("n0"),
                       dev.get("m0"), chunk=w.chunk, variant=w.variant, eps=1e-6, workspace=ws_f, out=fo)
        if do_bwd:
            tfla.mlstm_bwd(dev["q"], dev["k"], dev["v"], dev["i_pre"], dev["f_pre"], dev["dH"], fo["n_out"],
                           fo["m_out"], dev.get("C0"), dev.get("n0"), dev.get("m0"), None, chunk=w.chunk,
                           variant=w.variant, eps=1e-6, workspace=ws_b, out=bo,
                           fwd_workspace=None if args.recompute else ws_f)

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                      # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # Optionally the step (11 kernel launches of the two entry points) is captured once into a HIP
    # graph and the timed region replays it: same kernels, same work.  The library is capture-safe:
    # it never allocates, synchronises or records memset nodes.
    graph = None
    if args.graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
    run = graph.replay if graph is not None else step
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    # per-kernel durations: HIP events around every launch, in a separate eager pass over the same steps
    use_events = not args.no_kernel_events
    kernels, prof = {}, {}
    if use_events:
        tfla.profile_enable(16 * (args.steps + 1))
        torch.cuda.synchronize()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        prof = tfla.profile_read()
        tfla.profile_enable(0)
        kernels = {k_: v_["ms"] / v_["launches"] for k_, v_ in prof.items() if v_["launches"] > 0}

    tokens = w.B * w.T
    value = tokens / (ms_per_step * 1e-3)
    fl, fwd_fl, bwd_fl = algorithmic_flops(w)
    total_fl = fwd_fl + (bwd_fl if do_bwd else 0.0)
    peak = PEAK_BF16_MFMA if w.dtype == wl.BF16 else PEAK_FP32_MFMA

    roof = None
    if kernels and args.recompute:
        pass    # per-kernel roofline is reported for the default (workspace-reusing) step only
    elif kernels:
        es = 2 if w.dtype == wl.BF16 else 4
        byts = algorithmic_bytes(w, es)
        # a kernel symbol may be launched several times per step (the recurrent kernel runs forward,
        # forward again inside the backward call, and reversed): group the event families by symbol
        groups = {"recurrent_kernel": ["recurrent_fwd", "recurrent_bwd"], "tile_kernel<H>": ["tile_H"],
                  "tile_kernel<dV>": ["tile_dV"], "tile_kernel<dQ>": ["tile_dQ"], "tile_kernel<dK>": ["tile_dK"]}
        per = {}
        for sym, fams in groups.items():
            fams = [f for f in fams if f in prof and prof[f]["launches"] > 0]
            if not fams:
                continue
            n = sum(prof[f]["launches"] for f in fams)
            ms = sum(prof[f]["ms"] for f in fams)
            avg_s = ms / n * 1e-3
            flops = sum(fl[f] * prof[f]["launches"] for f in fams) / n
            bts = sum(byts[f] * prof[f]["launches"] for f in fams) / n
            per[sym] = {"launches_per_step": n / args.steps, "avg_ms": ms / n, "total_ms_per_step": ms / args.steps,
                        "flops": flops, "bytes": bts, "tflops": flops / avg_s / 1e12, "gbs": bts / avg_s / 1e9,
                        "mfma_frac": flops / avg_s / peak, "hbm_frac": bts / avg_s / PEAK_HBM}
        dom = max(per, key=lambda k_: per[k_]["total_ms_per_step"])
        pd = per[dom]
        # the roofline that binds a kernel is the one with the larger floor time
        hbm_bound = pd["bytes"] / PEAK_HBM > pd["flops"] / peak
        traffic = None
        if (w.name, w.chunk, w.variant) == ("c4", DEFAULT_CHUNK, wl.EXP):
            traffic = profiled_traffic().get(dom)
        roof = {"bound": "hbm" if hbm_bound else "mfma", "kernel": dom,
                "achieved": pd["gbs"] if hbm_bound else pd["tflops"],
                "peak": PEAK_HBM / 1e9 if hbm_bound else peak / 1e12,
                "unit": "GB/s" if hbm_bound else "TFLOP/s",
                "frac": pd["hbm_frac"] if hbm_bound else pd["mfma_frac"],
                "traffic": traffic,
                "traffic_source": "profiles/hbm_traffic_c4.txt (rocprofv3 --pmc runs of this command, not this run)" if traffic else None,
                "avg_launch_ms": pd["avg_ms"], "algorithmic_bytes_per_launch": pd["bytes"],
                "algorithmic_flops_per_launch": pd["flops"],
                "kernels": {k_: {m_: (round(x_, 5) if isinstance(x_, float) and x_ < 1e6 else x_) for m_, x_ in v_.items()}
                            for k_, v_ in per.items()},
                "kernel_ms": {k_: round(v_, 4) for k_, v_ in kernels.items()}}

    cpu = None
    if not args.no_cpu_baseline and not args.layer:
        from oracle import mlstm_oracle as orc
        nsl = min(16, w.B * w.NH)
        ds = wl.make_inputs(w, heads=nsl)
        oi = wl.oracle_inputs(ds)
        c0 = time.perf_counter()
        orc.recurrent_fwd(**oi, variant=w.variant, eps=1e-6)
        if do_bwd:
            orc.chunkwise_bwd(**oi, dH=wl.flat(ds["dH"]), variant=w.variant, eps=1e-6, chunk=w.chunk)
        c1 = time.perf_counter()
        frac = nsl / float(w.B * w.NH)
        cpu = {"value": tokens * frac / (c1 - c0), "unit": "tokens/s", "cores": int(orc.num_threads()),
               "kind": "oracle", "seconds": c1 - c0,
               "sample": "first %d of %d (batch, head) slices at full T: fp64 step-by-step recurrence forward%s; "
                         "tokens/s scaled by the slice fraction" % (nsl, w.B * w.NH,
                                                                   " + fp64 chunkwise backward (numpy)" if do_bwd else "")}

    line = {
        "metric": "mLSTM %s tokens/s and %% %s MFMA peak at T=%d, NH=%d, dqk=%d, dhv=%d" % (
            "fwd+bwd" if do_bwd else "fwd", "bf16" if w.dtype == wl.BF16 else "fp32", w.T, w.NH, w.dqk, w.dhv),
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == wl.BF16 else "f32", "data": "synthetic",
        "launch": "eager" if graph is None else "hip graph replay",
        "config": {"workload": w.name, "variant": "mLSTMexp" if w.variant == wl.EXP else "mLSTMsig",
                   "B": w.B, "NH": w.NH, "T": w.T, "dqk": w.dqk, "dhv": w.dhv, "chunk": w.chunk,
                   "tile_width": args.tile_width or "auto", "pass": ("layer " if args.layer else "") + ("fwd+bwd" if do_bwd else "fwd"), "states": "element type of q/k/v (bf16), fp32 accumulation"},
        "algorithmic_tflop_per_step": total_fl / 1e12,
        "mfma_frac_of_peak_whole_step": total_fl / (ms_per_step * 1e-3) / peak,
        "roofline": roof,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
