"""GPU parity at the edges of the supported range and in the degenerate cases of the method: one chunk only,
the smallest and the largest chunk and head dimensions, a (batch x head) count that is not a multiple of the
XCD count, gates that reset the memory at every step or never forget, a closed input gate, all-zero queries;
and two scalar-gate relatives evaluated through the same kernels (Sec. 5 related work: with the input gate fixed
to one and a constant decay the sigmoid-gate cell is decayed linear attention) against the textbook formula."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import mlstm_oracle as orc

pytestmark = pytest.mark.gpu


def _fwd_bwd(w, d, check_bwd=True, tol_scale=1.0, abs_tol=1e-4, df_scale_by_terms=False):
    import paper_2503_14376_amd as tfla
    from tests import gpu_util as gu
    dev = gu.dev_inputs(w, d)
    print("edge", w.variant, w.dtype, (w.B, w.NH, w.T, w.dqk, w.dhv, w.chunk), flush=True)
    f = tfla.mlstm_fwd(dev["q"], dev["k"], dev["v"], dev["i_pre"], dev["f_pre"], dev.get("C0"), dev.get("n0"),
                       dev.get("m0"), chunk=w.chunk, variant=w.variant, eps=1e-6)
    oi = gu.oracle_inputs(d)
    ref = orc.recurrent_fwd(**oi, variant=w.variant, eps=1e-6)
    tol = gu.TOL[w.dtype] * tol_scale
    errs = gu.check_fwd(w, d, f, ref, tol=tol, abs_tol=abs_tol)
    if check_bwd:
        b = tfla.mlstm_bwd(dev["q"], dev["k"], dev["v"], dev["i_pre"], dev["f_pre"], dev["dH"], f["n_out"], f["m_out"],
                           dev.get("C0"), dev.get("n0"), dev.get("m0"), None, chunk=w.chunk, variant=w.variant, eps=1e-6,
                           fwd_workspace=f["workspace"])
        torch.cuda.synchronize()
        rb = orc.chunkwise_bwd(**oi, dH=gu.flat(d["dH"]), variant=w.variant, eps=1e-6, chunk=min(w.chunk, 256))
        for key, rk in dict(dq="dq", dk="dk", dv="dv", d_i_pre="di", d_f_pre="df", dC0="dC0").items():
            ref_max = float(np.max(np.abs(rb[rk])))
            if ref_max < 1e-30:          # a gradient that is identically zero in exact arithmetic
                assert float(b[key].float().abs().max()) < 1e-20, key
                continue
            if key == "d_f_pre" and df_scale_by_terms:
                # Memory-reset cases only.  The forget-gate gradient is a cumulative sum over time of q_t.dq_t - k_t.dk_t
                # (what every gate pre-activation moves is the log-weight of the pairs it lies between).  When every
                # step forgets the past, those sums cancel to a gradient of order exp(-40): the error is then set by
                # the size of the terms, so the terms, not the cancelled result, are the scale it is measured against.
                qd = np.abs((oi["q"] * rb["dq"]).sum(-1)).max(); kd = np.abs((oi["k"] * rb["dk"]).sum(-1)).max()
                g_ = b[key].detach().float().cpu().numpy().astype(np.float64).reshape(rb[rk].shape)
                errs[key] = float(np.max(np.abs(g_ - rb[rk])) / max(ref_max, qd, kd))
            else:
                errs[key] = gu.rel_err(b[key], rb[rk])
            assert errs[key] <= tol, (key, errs)
    print("   ", errs, flush=True)
    return f, errs


@pytest.mark.parametrize("variant", [wl.EXP, wl.SIG])
@pytest.mark.parametrize("T,chunk", [(64, 64), (256, 256), (2048, 2048), (4096, 2048)])
def test_single_chunk_and_largest_chunk(variant, T, chunk):
    w = wl.small(variant, wl.BF16, B=1, NH=2, T=T, dqk=64, dhv=128, chunk=chunk, seed=71 + T)
    _fwd_bwd(w, wl.make_inputs(w))


@pytest.mark.parametrize("variant", [wl.EXP, wl.SIG])
@pytest.mark.parametrize("dqk,dhv", [(64, 64), (512, 512), (512, 64), (64, 512)])
def test_extreme_head_dimensions(variant, dqk, dhv):
    w = wl.small(variant, wl.BF16, B=1, NH=1, T=512, dqk=dqk, dhv=dhv, chunk=128, seed=73 + dqk + dhv)
    _fwd_bwd(w, wl.make_inputs(w))


@pytest.mark.parametrize("B,NH", [(1, 3), (5, 1), (3, 7)])
def test_batch_head_counts_not_multiple_of_eight(B, NH):
    w = wl.small(wl.EXP, wl.BF16, B=B, NH=NH, T=256, dqk=64, dhv=64, chunk=64, seed=75 + B)
    _fwd_bwd(w, wl.make_inputs(w))


@pytest.mark.parametrize("variant", [wl.EXP, wl.SIG])
@pytest.mark.parametrize("dtype", [wl.BF16, wl.F32])
@pytest.mark.parametrize("case", ["reset_every_step", "never_forget", "input_gate_closed", "zero_queries", "mixed_resets",
                                  "extreme_mix"])
def test_degenerate_gates(variant, dtype, case):
    w = wl.small(variant, dtype, B=1, NH=2, T=256, dqk=64, dhv=128, chunk=64, seed=77)
    d = wl.make_inputs(w)
    if case == "reset_every_step":        # f~ = -40: sigma(f~) ~ 4e-18, every step forgets the past
        d["f_pre"][:] = -40.0
    elif case == "never_forget":          # f~ = +40: log sigma(f~) = 0 in fp32, plain (normalised) linear attention
        d["f_pre"][:] = 40.0
    elif case == "input_gate_closed":     # i~ = -30 everywhere: only the initial state is visible
        d["i_pre"][:] = -30.0
    elif case == "zero_queries":
        d["q"][:] = 0.0
    elif case == "extreme_mix":           # |x| = 80 at scattered steps: exp(i~) ~ 5e34, resets next to saturated steps
        g = np.random.default_rng(78)
        for name in ("i_pre", "f_pre"):
            u = g.random(d[name].shape)
            d[name][u < 0.04] = -80.0
            d[name][u > 0.96] = 80.0
    else:                                  # resets at a few steps, open gates elsewhere
        d["f_pre"][:] = 6.0
        d["f_pre"][..., ::37] = -40.0
    # The max states and the weights are formed from cumulative sums of log sigma(f~) inside a chunk (App. B.2,
    # chunkwise gates): with f~ = -40 they reach -40 L = -2560, whose spacing in fp32 is 2.4e-4.  The fp32 kernels
    # therefore get their gate pre-pass in double and the two exponents of a weight as (rounded, remainder) pairs, and
    # hold the stated 1e-4 here too; on the bf16 path (bar 2e-2) the max states of the reset cases, which cancel from
    # two numbers of that size, are compared at 1e-3 absolute.
    resets = case in ("reset_every_step", "mixed_resets")
    _fwd_bwd(w, d, abs_tol=1e-3 if (resets and dtype == wl.BF16) else 1e-4, df_scale_by_terms=resets)


def test_relatives_through_the_same_kernel():
    """Input gate fixed to one and one constant decay per head: h_t = sum_{j<=t} gamma^(t-j) (q_t.k_j/sqrt(d)) v_j,
    the retention / simple gated-linear-attention form, evaluated by the mLSTMsig kernels (i~ = +40, f~ = logit gamma)
    and compared with that formula written out in numpy."""
    import paper_2503_14376_amd as tfla
    from tests import gpu_util as gu
    B, NH, T, dqk, dhv = 1, 4, 256, 64, 128
    w = wl.small(wl.SIG, wl.F32, B=B, NH=NH, T=T, dqk=dqk, dhv=dhv, chunk=64, seed=79, init_state=False)
    d = wl.make_inputs(w)
    gammas = np.array([0.5, 0.9, 0.97, 0.995])
    d["i_pre"][:] = 40.0
    d["f_pre"][:] = np.log(gammas / (1 - gammas)).astype(np.float32)[None, :, None]
    dev = gu.dev_inputs(w, d)
    f = tfla.mlstm_fwd(dev["q"], dev["k"], dev["v"], dev["i_pre"], dev["f_pre"], chunk=64, variant=wl.SIG)
    torch.cuda.synchronize()
    t = np.arange(T)
    for h in range(NH):
        g_eff = 1.0 / (1.0 + np.exp(-np.float64(d["f_pre"][0, h, 0])))
        decay = np.tril(g_eff ** (t[:, None] - t[None, :]).clip(min=0))
        S = (d["q"][0, h].astype(np.float64) @ d["k"][0, h].astype(np.float64).T) / np.sqrt(dqk) * decay
        ref = S @ d["v"][0, h].astype(np.float64)
        assert gu.rel_err(f["H"][0, h], ref) <= 1e-4, h


@pytest.mark.parametrize("dtype", [wl.BF16, wl.F32])
@pytest.mark.parametrize("relative", ["decay_only", "input_gate_only", "plain_linear_attention"])
def test_relatives_forward_and_backward(dtype, relative):
    """The scalar-gate relatives of Sec. 5 / App. A.2 through the mLSTMsig entry points, forward and backward, in both
    element types, against the fp64 oracle on the same gate values: a constant decay per head with the input gate
    fixed to one (retention / simple gated linear attention), a data-dependent input gate without forgetting, and
    no gates at all (causal linear attention).  A gate "fixed to one" is a pre-activation of +40 (sigma = 1 to fp32
    precision); its gradient is then of order sigma(-40) and is compared like any other output."""
    w = wl.small(wl.SIG, dtype, B=1, NH=4, T=512, dqk=128, dhv=128, chunk=128, seed=83, init_state=False)
    d = wl.make_inputs(w)
    if relative == "decay_only":
        gammas = np.array([0.5, 0.9, 0.97, 0.995])
        d["i_pre"][:] = 40.0
        d["f_pre"][:] = np.log(gammas / (1 - gammas)).astype(np.float32)[None, :, None]
    elif relative == "input_gate_only":
        d["f_pre"][:] = 40.0
    else:
        d["i_pre"][:] = 40.0
        d["f_pre"][:] = 40.0
        # without decay the sums grow with t: scale the values so that bf16 outputs stay well inside the format
        d["v"] = wl.bf16_round(d["v"] * np.float32(0.25)) if dtype == wl.BF16 else d["v"] * np.float32(0.25)
    _fwd_bwd(w, d)


@pytest.mark.parametrize("variant", [wl.EXP, wl.SIG])
@pytest.mark.parametrize("dtype", [wl.BF16, wl.F32])
@pytest.mark.parametrize("T,chunk", [(1, 64), (63, 64), (100, 64), (200, 64), (449, 128), (1000, 256)])
def test_ragged_sequence_length(variant, dtype, T, chunk):
    """T is not a multiple of the chunk (N_c = ceil(T / L), Sec. 2.2): outputs, final state and all gradients are those
    of the T-step sequence (the oracle's recurrence and its ragged last chunk know nothing of padding)."""
    import paper_2503_14376_amd as tfla
    from tests import gpu_util as gu
    w = wl.small(variant, dtype, B=2, NH=2, T=T, dqk=64, dhv=128, chunk=chunk, seed=81 + T)
    d = wl.make_inputs(w)
    f, _ = _fwd_bwd(w, d, check_bwd=T > 1)
    if T >= 100:
        # continuation: the returned state is the state after step T, not after the padded chunk
        T1 = T - 37
        cut = lambda a, lo, hi: np.ascontiguousarray(a[:, :, lo:hi])
        dev = gu.dev_inputs(w, d)
        sl = lambda key, lo, hi: dev[key][:, :, lo:hi].contiguous()
        a = tfla.mlstm_fwd(sl("q", 0, T1), sl("k", 0, T1), sl("v", 0, T1), sl("i_pre", 0, T1), sl("f_pre", 0, T1),
                           dev.get("C0"), dev.get("n0"), dev.get("m0"), chunk=chunk, variant=variant, eps=1e-6)
        b = tfla.mlstm_fwd(sl("q", T1, T), sl("k", T1, T), sl("v", T1, T), sl("i_pre", T1, T), sl("f_pre", T1, T),
                           a["Cn"], a["nn"] if variant == wl.EXP else None, a["mn"] if variant == wl.EXP else None,
                           chunk=chunk, variant=variant, eps=1e-6)
        torch.cuda.synchronize()
        ref = orc.recurrent_fwd(**gu.oracle_inputs(d), variant=variant, eps=1e-6)
        tol = gu.TOL[dtype]
        assert gu.rel_err(b["H"], ref["H"][:, T1:].reshape(2, 2, T - T1, -1)) <= tol
        assert gu.rel_err(b["Cn"], ref["Cn"]) <= tol


def test_ragged_layer():
    from tests.test_gpu_layer import run_layer
    from oracle import layer_oracle as lo
    w = wl.small(wl.EXP, wl.BF16, B=2, NH=2, T=300, dqk=64, dhv=128, chunk=128, seed=83, init_state=False)
    run_layer(w, lo.LAYER, softcap=15.0, gate=True, gate_scale=2.0, chunk_oracle=50)


def test_zero_batch_is_an_error_not_a_launch():
    import paper_2503_14376_amd as tfla
    assert tfla.check(0, 0, 8, 256, 64, 64, 64, 0, 1) == -2
    assert tfla.check(0, 1, 8, 0, 64, 64, 64, 0, 1) == -2


@pytest.mark.parametrize("variant", [wl.EXP, wl.SIG])
@pytest.mark.parametrize("dtype", [wl.BF16, wl.F32])
@pytest.mark.parametrize("dqk,dhv,T", [(32, 32, 256), (96, 192, 320), (192, 80, 200), (8, 64, 128), (256, 384, 256)])
def test_head_dimensions_between_the_kernel_widths(variant, dtype, dqk, dhv, T):
    """Head dimensions that are not 64, 128, 256 or 512 (the paper's head-dimension benchmark starts at 32): forward
    with an initial state, final state, backward -- everything as for the problem as given, 1/sqrt(dqk) of the true dqk
    included."""
    w = wl.small(variant, dtype, B=1, NH=2, T=T, dqk=dqk, dhv=dhv, chunk=64, seed=85 + dqk + dhv)
    _fwd_bwd(w, wl.make_inputs(w))


@pytest.mark.parametrize("variant", [wl.EXP, wl.SIG])
@pytest.mark.parametrize("dqk,dhv,chunk", [(512, 512, 64), (256, 512, 128), (512, 64, 64)])
def test_fp32_head_dimensions_up_to_512(variant, dqk, dhv, chunk):
    """fp32 with 512-wide heads: a contraction over 512 fp32 columns runs as two 256-wide launches that meet in fp32
    (H and dV when dqk = 512, dQ and dK when dhv = 512).  Initial state, final state, backward, 1e-4."""
    w = wl.small(variant, wl.F32, B=1, NH=2, T=256, dqk=dqk, dhv=dhv, chunk=chunk, seed=89 + dqk + dhv)
    _fwd_bwd(w, wl.make_inputs(w))


_SWEEP = [(dqk, dhv, chunk) for dqk in (64, 128, 256, 512) for dhv in (64, 128, 256, 512) for chunk in (64, 128, 192, 256)
          if (dqk * 3 + dhv * 5 + chunk * 7) % 5 in (0, 2)]       # a fixed two-fifths of the 64 combinations


@pytest.mark.parametrize("dqk,dhv,chunk", _SWEEP)
def test_kernel_width_and_chunk_combinations(dqk, dhv, chunk):
    """Every kernel width with every kind of chunk size (multiples of 128 take the four-wavefront workgroups and the
    128-row pieces, the others the two-wavefront ones and 64-row pieces): forward with initial state and backward."""
    variant = wl.EXP if (dqk + dhv + chunk) % 128 == 0 else wl.SIG
    w = wl.small(variant, wl.BF16, B=1, NH=2, T=3 * chunk, dqk=dqk, dhv=dhv, chunk=chunk, seed=87 + dqk + dhv + chunk)
    _fwd_bwd(w, wl.make_inputs(w))


@pytest.mark.parametrize("dqk,dhv,chunk", [(64, 256, 64), (128, 64, 192), (256, 256, 128), (256, 128, 64), (64, 64, 256),
                                           (128, 256, 192), (256, 64, 128)])
def test_kernel_width_and_chunk_combinations_fp32(dqk, dhv, chunk):
    variant = wl.EXP if (dqk + chunk) % 128 == 0 else wl.SIG
    w = wl.small(variant, wl.F32, B=1, NH=2, T=2 * chunk, dqk=dqk, dhv=dhv, chunk=chunk, seed=89 + dqk + dhv + chunk)
    _fwd_bwd(w, wl.make_inputs(w))


def test_more_than_65536_chunk_workgroup_groups():
    """batch*head x chunks beyond what one grid dimension holds (the tiled kernels are launched on a one-dimensional
    grid): the first and the last (batch, head) slice against the oracle, forward and backward."""
    import paper_2503_14376_amd as tfla
    from tests import gpu_util as gu
    B, NH, T, d, chunk = 128, 8, 4096, 64, 64           # 1024 slices x 64 chunks = 65536
    g = torch.Generator(device="cuda").manual_seed(4242)
    bf = torch.bfloat16
    mk = lambda *shape: torch.randn(shape, device="cuda", generator=g)
    q, k, v, dH = (mk(B, NH, T, d).to(bf) for _ in range(4))
    ip, fp = mk(B, NH, T), mk(B, NH, T) + 3.0
    print("edge big grid", (B, NH, T, d, chunk), flush=True)
    f = tfla.mlstm_fwd(q, k, v, ip, fp, chunk=chunk, variant=wl.EXP, eps=1e-6)
    b = tfla.mlstm_bwd(q, k, v, ip, fp, dH, f["n_out"], f["m_out"], chunk=chunk, variant=wl.EXP, eps=1e-6,
                       fwd_workspace=f["workspace"])
    torch.cuda.synchronize()
    for (bi, hi) in ((0, 0), (B - 1, NH - 1), (77, 3)):
        sl = lambda t: t[bi, hi].float().cpu().numpy().astype(np.float64)[None]
        ref = orc.recurrent_fwd(sl(q), sl(k), sl(v), sl(ip), sl(fp), variant=wl.EXP, eps=1e-6)
        rb = orc.chunkwise_bwd(sl(q), sl(k), sl(v), sl(ip), sl(fp), sl(dH), variant=wl.EXP, eps=1e-6, chunk=256)
        assert gu.rel_err(f["H"][bi, hi], ref["H"][0]) <= 2e-2
        assert gu.rel_err(f["Cn"][bi, hi], ref["Cn"][0]) <= 2e-2
        for key, rk in dict(dq="dq", dk="dk", dv="dv", d_i_pre="di", d_f_pre="df").items():
            assert gu.rel_err(b[key][bi, hi], rb[rk][0]) <= 2e-2, (bi, hi, key)


@pytest.mark.parametrize("variant", [wl.EXP, wl.SIG])
def test_optional_outputs_may_be_omitted(variant):
    """No final state, no n/m record, no dC0: through the C ABI with NULL pointers; what is produced equals the full call."""
    import ctypes
    import paper_2503_14376_amd as tfla
    from paper_2503_14376_amd import binding as bd
    from tests import gpu_util as gu
    w = wl.small(variant, wl.BF16, B=1, NH=2, T=256, dqk=64, dhv=128, chunk=64, seed=95, init_state=False)
    dev = gu.dev_inputs(w, wl.make_inputs(w))
    full = tfla.mlstm_fwd(dev["q"], dev["k"], dev["v"], dev["i_pre"], dev["f_pre"], chunk=64, variant=variant)
    gfull = tfla.mlstm_bwd(dev["q"], dev["k"], dev["v"], dev["i_pre"], dev["f_pre"], dev["dH"], full["n_out"], full["m_out"],
                           chunk=64, variant=variant)
    lib = tfla.load_library()
    P = bd._ptr
    H = torch.empty_like(full["H"])
    ws = torch.empty(tfla.workspace_bytes(0, 1, 2, 256, 64, 128, 64, variant, 1), dtype=torch.uint8, device="cuda")
    rc = lib.tfla_mlstm_fwd(P(dev["q"]), P(dev["k"]), P(dev["v"]), P(dev["i_pre"]), P(dev["f_pre"]), None, None, None,
                            1, 2, 256, 64, 128, 64, variant, 1, 1e-6, P(H), None, None, None, None, None,
                            P(ws), ws.numel(), bd._stream_handle(None))
    assert rc == 0
    torch.cuda.synchronize()
    assert torch.equal(H, full["H"])
    g = tfla.mlstm_bwd(dev["q"], dev["k"], dev["v"], dev["i_pre"], dev["f_pre"], dev["dH"], full["n_out"], full["m_out"],
                       chunk=64, variant=variant, want_dC0=False)
    torch.cuda.synchronize()
    assert "dC0" not in g
    for key in ("dq", "dk", "dv", "d_i_pre", "d_f_pre"):
        assert torch.equal(g[key], gfull[key]), key


@pytest.mark.parametrize("variant", [wl.EXP, wl.SIG])
@pytest.mark.parametrize("dqk,dhv,chunk", [(1024, 1024, 256), (1024, 1024, 64), (512, 1024, 128), (1024, 256, 192),
                                           (64, 1024, 64), (1024, 64, 256)])
def test_head_dimensions_up_to_1024(variant, dqk, dhv, chunk):
    """Head dimensions above 512 (the head-dimension benchmark of App. E.3 ends at 1024): the tiled kernels contract
    over a 1024-wide dimension in two halves that meet in fp32; initial state given, so that every term is present."""
    w = wl.small(variant, wl.BF16, B=1, NH=2, T=576 if chunk == 192 else 512, dqk=dqk, dhv=dhv, chunk=chunk,
                 seed=300 + dqk // 64 + dhv // 8 + chunk)
    _fwd_bwd(w, wl.make_inputs(w))


@pytest.mark.parametrize("variant", [wl.EXP, wl.SIG])
def test_head_dimensions_between_512_and_1024_and_ragged_length(variant):
    w = wl.small(variant, wl.BF16, B=1, NH=1, T=300, dqk=520, dhv=1000, chunk=128, seed=411)
    _fwd_bwd(w, wl.make_inputs(w))


@pytest.mark.parametrize("width", [64, 128])
def test_tile_width_override_gives_the_same_results(width):
    """The tile-size sweep's knob: every block width the kernels are built with gives results within tolerance, at the
    benchmark's head shape (where the automatic choice is 128 for H / dV and 256 for dQ / dK)."""
    import paper_2503_14376_amd as tfla
    w = wl.small(wl.EXP, wl.BF16, B=1, NH=2, T=512, dqk=256, dhv=512, chunk=256, seed=97)
    tfla.tile_width(width)
    try:
        _fwd_bwd(w, wl.make_inputs(w))
    finally:
        tfla.tile_width(0)


def test_sigmoid_variant_zero_fills_the_outputs_it_does_not_have():
    """mLSTMsig has no normaliser and no max state: nn, mn, n_out, m_out come back as zeros (one fill launch for
    all of them), whatever the buffers held before; likewise n and m of the generation step."""
    import paper_2503_14376_amd as tfla
    from tests import gpu_util as gu
    w = wl.small(wl.SIG, wl.BF16, B=2, NH=3, T=192, dqk=64, dhv=128, chunk=64, seed=99)
    dev = gu.dev_inputs(w, wl.make_inputs(w))
    call = lambda out: tfla.mlstm_fwd(dev["q"], dev["k"], dev["v"], dev["i_pre"], dev["f_pre"], dev.get("C0"), None, None,
                                      chunk=w.chunk, variant=w.variant, eps=1e-6, out=out)
    out = {}
    call(out)
    for key in ("nn", "mn", "n_out", "m_out"):
        out[key].fill_(float("nan"))
    call(out)
    torch.cuda.synchronize()
    for key in ("nn", "mn", "n_out", "m_out"):
        assert float(out[key].abs().max()) == 0.0, key
    s = tfla.mlstm_step(dev["q"][:, :, 0].contiguous(), dev["k"][:, :, 0].contiguous(), dev["v"][:, :, 0].contiguous(),
                        dev["i_pre"][:, :, 0].contiguous(), dev["f_pre"][:, :, 0].contiguous(), out["Cn"], None, None,
                        variant=w.variant)
    s["n"].fill_(float("nan")); s["m"].fill_(float("nan"))
    s2 = tfla.mlstm_step(dev["q"][:, :, 0].contiguous(), dev["k"][:, :, 0].contiguous(), dev["v"][:, :, 0].contiguous(),
                         dev["i_pre"][:, :, 0].contiguous(), dev["f_pre"][:, :, 0].contiguous(), out["Cn"], None, None,
                         variant=w.variant, out=s)
    torch.cuda.synchronize()
    assert float(s2["n"].abs().max()) == 0.0 and float(s2["m"].abs().max()) == 0.0
