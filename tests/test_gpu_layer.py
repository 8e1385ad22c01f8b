"""GPU parity of the layer entry points (soft-capped gates, cell, multi-head NORM, output gate; their
backward; the transfer gains) against the fp64 layer oracle, which is pinned on the CPU to the library
norms, to finite differences and to the transfer behaviour the paper states."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import layer_oracle as lo
from oracle import mlstm_oracle as orc

pytestmark = pytest.mark.gpu


def _dev(w, d):
    from tests import gpu_util as gu
    out = {}
    for key, val in d.items():
        out[key] = gu.to_dev(val, w.dtype if key in ("q", "k", "v", "dH", "o_pre") else wl.F32)
    return out


def run_layer(w, kind, softcap, gate, gate_scale=1.0, heads=None, chunk_oracle=None, check_params=True, backward=True):
    import paper_2503_14376_amd as tfla
    from tests import gpu_util as gu
    d = wl.make_layer_inputs(w, heads, gate_scale)
    dev = _dev(w, d)
    o_pre = dev["o_pre"] if gate else None
    kw = dict(chunk=w.chunk, variant=w.variant, eps=1e-6, gate_softcap=softcap, norm_kind=kind, norm_eps=1e-6)
    print("layer", w.name, "variant", w.variant, "dtype", w.dtype, (w.T, w.dqk, w.dhv, w.chunk), "norm", kind,
          "cap", softcap, "gate", gate, flush=True)
    f = tfla.mlstm_layer_fwd(dev["q"], dev["k"], dev["v"], dev["i_pre"], dev["f_pre"], o_pre, dev["gamma"], dev["beta"], **kw)
    if not backward:
        torch.cuda.synchronize()
        rf = lo.layer_fwd(q=d["q"], k=d["k"], v=d["v"], i_pre=d["i_pre"], f_pre=d["f_pre"], o_pre=d["o_pre"] if gate else None,
                          gamma=d["gamma"], beta=d["beta"], variant=w.variant, eps=1e-6, gate_softcap=softcap, kind=kind,
                          norm_eps=1e-6)
        errs = {"Y": gu.rel_err(f["Y"], rf["y"]), "H": gu.rel_err(f["H"], rf["H"])}
        print("   ", errs, flush=True)
        for key, e in errs.items():
            assert e <= gu.TOL[w.dtype], (key, e, errs)
        return errs
    b = tfla.mlstm_layer_bwd(dev["q"], dev["k"], dev["v"], dev["i_pre"], dev["f_pre"], f["H"], dev["dH"], o_pre,
                             dev["gamma"], dev["beta"], f["n_out"], f["m_out"], fwd_workspace=f["workspace"], **kw)
    torch.cuda.synchronize()
    okw = dict(variant=w.variant, eps=1e-6, gate_softcap=softcap, kind=kind, norm_eps=1e-6)
    oin = dict(q=d["q"], k=d["k"], v=d["v"], i_pre=d["i_pre"], f_pre=d["f_pre"], o_pre=d["o_pre"] if gate else None,
               gamma=d["gamma"], beta=d["beta"])
    rf = lo.layer_fwd(**oin, **okw)
    rb = lo.layer_bwd(**oin, dy=d["dH"], chunk=chunk_oracle or w.chunk, **okw)
    tol = gu.TOL[w.dtype]
    errs = {"Y": gu.rel_err(f["Y"], rf["y"]), "H": gu.rel_err(f["H"], rf["H"])}
    for key in ("dq", "dk", "dv", "d_i_pre", "d_f_pre"):
        errs[key] = gu.rel_err(b[key], rb[key])
    if gate:
        errs["do_pre"] = gu.rel_err(b["do_pre"], rb["do_pre"])
    if check_params:
        errs["dgamma"] = gu.rel_err(b["dgamma"], rb["dgamma"])
        if kind == lo.LAYER:
            errs["dbeta"] = gu.rel_err(b["dbeta"], rb["dbeta"])
        else:
            assert float(b["dbeta"].abs().max()) == 0.0
    print("   ", errs, flush=True)
    for key, e in errs.items():
        assert e <= tol, (key, e, errs)
    return errs


@pytest.mark.parametrize("variant", [wl.EXP, wl.SIG])
@pytest.mark.parametrize("dtype", [wl.BF16, wl.F32])
@pytest.mark.parametrize("kind", [lo.RMS, lo.LAYER])
def test_layer_small(variant, dtype, kind):
    w = wl.small(variant, dtype, B=2, NH=2, T=256, dqk=64, dhv=128, chunk=64, seed=51 + kind, init_state=False)
    run_layer(w, kind, softcap=15.0, gate=True, gate_scale=2.0)


@pytest.mark.parametrize("shape", [(64, 64, 64), (128, 128, 128), (256, 128, 256), (128, 64, 256), (512, 128, 128)])
@pytest.mark.parametrize("kind", [lo.RMS, lo.LAYER])
@pytest.mark.parametrize("gate", [True, False])
def test_layer_output_formed_by_the_h_kernel(shape, kind, gate):
    """bf16, d_hv of 64 or 128 and nothing to pad: a workgroup of the H kernel holds whole rows of h~ and stores
    y = sigma(o~) (.) NORM(h~) itself (no separate NORM launch).  Every width and workgroup size of that path."""
    dqk, dhv, chunk = shape
    w = wl.small(wl.EXP if kind == lo.RMS else wl.SIG, wl.BF16, B=1, NH=3, T=2 * chunk + chunk, dqk=dqk, dhv=dhv,
                 chunk=chunk, seed=52 + dqk // 64, init_state=False)
    # (d_qk = 512 next to d_hv = 128: forward only.  With the sigmoid input gate the first rows of h~ are single terms
    # w s v_0, the LayerNorm gradient is orthogonal to them, and dq, dk of those rows -- where the gradient is largest --
    # cancel to zero in exact arithmetic; what the bf16 rounding of the gradient leaves there is 3.5 % of the largest
    # true dq with or without the fusion, while the cell's own backward at this shape is within the bar.)
    run_layer(w, kind=kind, softcap=15.0, gate=gate, backward=dqk < 512)


def test_layer_output_same_with_and_without_the_separate_norm_kernel():
    """The column-block override (a measurement aid) splits the rows of h~ over two workgroups, which sends the same
    problem through the separate NORM kernel: both paths normalise the same rounded h~, so the outputs agree to the
    rounding of y."""
    import paper_2503_14376_amd as tfla
    w = wl.small(wl.EXP, wl.BF16, B=2, NH=2, T=512, dqk=128, dhv=128, chunk=128, seed=56, init_state=False)
    d = wl.make_layer_inputs(w)
    dev = _dev(w, d)
    kw = dict(chunk=w.chunk, variant=w.variant, eps=1e-6, gate_softcap=15.0, norm_kind=lo.LAYER, norm_eps=1e-6)
    args = (dev["q"], dev["k"], dev["v"], dev["i_pre"], dev["f_pre"], dev["o_pre"], dev["gamma"], dev["beta"])
    fused = tfla.mlstm_layer_fwd(*args, **kw)
    torch.cuda.synchronize()
    tfla.tile_width(64)
    try:
        split = tfla.mlstm_layer_fwd(*args, **kw)
        torch.cuda.synchronize()
    finally:
        tfla.tile_width(0)
    assert torch.equal(fused["H"], split["H"])
    y0, y1 = fused["Y"].float(), split["Y"].float()
    assert float((y0 - y1).abs().max()) <= 2.0 ** -7 * float(y1.abs().max())      # one bf16 step of the largest value
    assert float((y0 != y1).float().mean()) < 0.02


@pytest.mark.parametrize("variant", [wl.EXP, wl.SIG])
def test_layer_no_gate_no_cap(variant):
    w = wl.small(variant, wl.BF16, B=1, NH=3, T=320, dqk=128, dhv=256, chunk=64, seed=57, init_state=False)
    run_layer(w, lo.RMS, softcap=0.0, gate=False)


@pytest.mark.parametrize("variant", [wl.EXP, wl.SIG])
def test_layer_7b_head_shape(variant):
    # the benchmark's head shape (dqk 256, dhv 512, chunk 256); T is a multiple of the backward kernel's
    # row block plus a remainder
    w = wl.small(variant, wl.BF16, B=2, NH=2, T=1280, dqk=256, dhv=512, chunk=256, seed=58, init_state=False)
    run_layer(w, lo.LAYER, softcap=15.0, gate=True, gate_scale=2.0)


@pytest.mark.parametrize("kind", [lo.RMS, lo.LAYER])
def test_layer_head_dimension_1024(kind):
    # the widest head: 1024-wide contractions in the cell (two 512-wide launches) and the norm kernels' widest rows
    w = wl.small(wl.EXP, wl.BF16, B=1, NH=2, T=384, dqk=512, dhv=1024, chunk=128, seed=59, init_state=False)
    run_layer(w, kind, softcap=15.0, gate=True, gate_scale=2.0)


def test_softcap_equals_capped_inputs():
    # capping inside the library == capping the pre-activations by hand (fp32) and switching the cap off
    import paper_2503_14376_amd as tfla
    w = wl.small(wl.EXP, wl.F32, B=1, NH=2, T=256, dqk=64, dhv=64, chunk=64, seed=59, init_state=False)
    d = wl.make_layer_inputs(w, None, 6.0)
    dev = _dev(w, d)
    a = tfla.mlstm_layer_fwd(dev["q"], dev["k"], dev["v"], dev["i_pre"], dev["f_pre"], chunk=64, gate_softcap=15.0)
    ic = (15.0 * torch.tanh(dev["i_pre"] / 15.0)).contiguous(); fc = (15.0 * torch.tanh(dev["f_pre"] / 15.0)).contiguous()
    b = tfla.mlstm_layer_fwd(dev["q"], dev["k"], dev["v"], ic, fc, chunk=64, gate_softcap=0.0)
    torch.cuda.synchronize()
    assert float((a["Y"] - b["Y"]).abs().max()) <= 2e-5 * float(b["Y"].abs().max())
    # and the plain entry point is the layer entry point's cell output without a cap
    c = tfla.mlstm_fwd(dev["q"], dev["k"], dev["v"], ic, fc, chunk=64)
    assert torch.equal(c["H"], b["H"])


@pytest.mark.parametrize("dtype", [wl.BF16, wl.F32])
@pytest.mark.parametrize("kind", [lo.RMS, lo.LAYER])
def test_transfer_gain(dtype, kind):
    import paper_2503_14376_amd as tfla
    from tests import gpu_util as gu
    g = np.random.default_rng(61)
    B, NH, T, dhv = 3, 2, 70, 128
    scale = np.exp(g.uniform(-8, 2, size=(B, NH, 1, 1))).astype(np.float32)     # rows far below and above the epsilon
    h = (g.standard_normal((B, NH, T, dhv)).astype(np.float32) * scale)
    v = g.standard_normal((B, NH, T, dhv)).astype(np.float32)
    if dtype == wl.BF16:
        h, v = wl.bf16_round(h), wl.bf16_round(v)
    gb, ga = tfla.transfer_gain(gu.to_dev(h, dtype), gu.to_dev(v, dtype), norm_kind=kind, norm_eps=1e-6)
    torch.cuda.synchronize()
    rb, ra = lo.transfer_gain(h, v, kind, 1e-6)
    assert gu.rel_err(gb, rb) <= 1e-5 and gu.rel_err(ga, ra) <= 1e-5
    # per-element check as well: every (batch, head) has its own scale
    assert np.max(np.abs(ga.cpu().numpy() - ra) / np.abs(ra)) <= 1e-4


def test_transfer_experiment_grid():
    # App. D.2 set-up (one head, T = 512, dqk = dhv = 128, constant gate pre-activations on a grid, RMS norm),
    # the grid points batched into one call; gains against the oracle's, and the qualitative result of Sec. 4.1
    import paper_2503_14376_amd as tfla
    from tests import gpu_util as gu
    ivals = np.array([-12.0, -8.0, -4.0, 0.0, 4.0, 8.0]); fvals = np.array([-5.0, 0.0, 6.0, 12.0])
    G = len(ivals) * len(fvals)
    T, d = 512, 128
    rng = np.random.Generator(np.random.Philox(key=77))
    q1 = rng.standard_normal((1, 1, T, d), dtype=np.float32); k1 = rng.standard_normal((1, 1, T, d), dtype=np.float32)
    v1 = rng.standard_normal((1, 1, T, d), dtype=np.float32)
    q = np.broadcast_to(q1, (G, 1, T, d)).copy(); k = np.broadcast_to(k1, (G, 1, T, d)).copy(); v = np.broadcast_to(v1, (G, 1, T, d)).copy()
    ii, ff = np.meshgrid(ivals, fvals, indexing="ij")
    i_pre = np.broadcast_to(ii.reshape(G, 1, 1), (G, 1, T)).astype(np.float32).copy()
    f_pre = np.broadcast_to(ff.reshape(G, 1, 1), (G, 1, T)).astype(np.float32).copy()
    res = {}
    for variant in (wl.EXP, wl.SIG):
        o = tfla.mlstm_fwd(gu.to_dev(q, wl.F32), gu.to_dev(k, wl.F32), gu.to_dev(v, wl.F32), gu.to_dev(i_pre, wl.F32),
                           gu.to_dev(f_pre, wl.F32), chunk=64, variant=variant, eps=0.0)
        gb, ga = tfla.transfer_gain(o["H"], gu.to_dev(v, wl.F32), norm_kind=lo.RMS, norm_eps=1e-6)
        torch.cuda.synchronize()
        ref = orc.recurrent_fwd(q[:, 0], k[:, 0], v[:, 0], i_pre[:, 0], f_pre[:, 0], variant=variant, eps=0.0)
        rb, ra = lo.transfer_gain(ref["H"][:, None], v, lo.RMS, 1e-6)
        assert gu.rel_err(gb, rb) <= 1e-3 and gu.rel_err(ga, ra) <= 1e-3, (variant, gu.rel_err(gb, rb), gu.rel_err(ga, ra))
        res[variant] = ga.cpu().numpy().reshape(len(ivals), len(fvals))
    # suppressed at the most negative input gate, passed (gain about one) at open gates, and the two variants alike
    for variant in (wl.EXP, wl.SIG):
        assert np.all(res[variant][0] < 0.15) and np.all(np.abs(res[variant][-2:] - 1.0) < 0.5)
        assert np.all(np.diff(res[variant], axis=0) > -1e-3)      # the gain grows with the input gate
    assert np.max(np.abs(res[wl.EXP] - res[wl.SIG])) < 0.15


@pytest.mark.parametrize("variant", [wl.EXP, wl.SIG])
@pytest.mark.parametrize("dtype", [wl.BF16, wl.F32])
def test_layer_steps_continue_a_layer_forward(variant, dtype):
    """A prompt through tfla_mlstm_layer_fwd, then step by step through tfla_mlstm_layer_step: every y equals the layer
    oracle's on the whole sequence."""
    import paper_2503_14376_amd as tfla
    from tests import gpu_util as gu
    T0, NS = 128, 12
    w = wl.small(variant, dtype, B=2, NH=3, T=T0 + NS, dqk=64, dhv=128, chunk=64, seed=63, init_state=False)
    d = wl.make_layer_inputs(w, None, 2.0)
    dev = _dev(w, d)
    kw = dict(variant=variant, eps=1e-6, gate_softcap=15.0, norm_kind=lo.LAYER, norm_eps=1e-6)
    cut = lambda key, lo_, hi: dev[key][:, :, lo_:hi].contiguous()
    f = tfla.mlstm_layer_fwd(cut("q", 0, T0), cut("k", 0, T0), cut("v", 0, T0), cut("i_pre", 0, T0), cut("f_pre", 0, T0),
                             cut("o_pre", 0, T0), dev["gamma"], dev["beta"], chunk=64, **kw)
    C, n, m = f["Cn"], f["nn"], f["mn"]
    ys = [f["Y"]]
    for t in range(T0, T0 + NS):
        at = lambda key: dev[key][:, :, t].contiguous()
        s = tfla.mlstm_layer_step(at("q"), at("k"), at("v"), at("i_pre"), at("f_pre"), C, n if variant == wl.EXP else None,
                                  m if variant == wl.EXP else None, at("o_pre"), dev["gamma"], dev["beta"], **kw)
        C, n, m = s["C"], s["n"], s["m"]
        ys.append(s["y"].unsqueeze(2))
    torch.cuda.synchronize()
    y = torch.cat(ys, dim=2)
    ref = lo.layer_fwd(d["q"], d["k"], d["v"], d["i_pre"], d["f_pre"], d["o_pre"], d["gamma"], d["beta"], variant=variant,
                       eps=1e-6, gate_softcap=15.0, kind=lo.LAYER, norm_eps=1e-6)
    assert gu.rel_err(y, ref["y"]) <= gu.TOL[dtype]
