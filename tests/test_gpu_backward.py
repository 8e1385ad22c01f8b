"""GPU parity of tfla_mlstm_bwd against the fp64 oracle (chunkwise backward of App. B.3, itself
pinned to the frozen-normaliser definition and to finite differences on the CPU)."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import mlstm_oracle as orc

pytestmark = pytest.mark.gpu


def run_case(w, with_dCn=False, heads=None, oracle_chunk=None):
    import paper_2503_14376_amd as tfla
    from tests import gpu_util as gu
    d = wl.make_inputs(w, heads)
    dev = gu.dev_inputs(w, d)
    S = d["q"].shape[0] * d["q"].shape[1]
    dCn_np = None
    if with_dCn:
        g = np.random.default_rng(w.seed + 99)
        dCn_np = g.standard_normal((d["q"].shape[0], d["q"].shape[1], w.dqk, w.dhv)).astype(np.float32)
    dCn = None if dCn_np is None else torch.from_numpy(dCn_np).cuda()
    fwd = tfla.mlstm_fwd(dev["q"], dev["k"], dev["v"], dev["i_pre"], dev["f_pre"],
                         dev.get("C0"), dev.get("n0"), dev.get("m0"), chunk=w.chunk, variant=w.variant, eps=1e-6)
    out = tfla.mlstm_bwd(dev["q"], dev["k"], dev["v"], dev["i_pre"], dev["f_pre"], dev["dH"],
                         fwd["n_out"], fwd["m_out"], dev.get("C0"), dev.get("n0"), dev.get("m0"), dCn,
                         chunk=w.chunk, variant=w.variant, eps=1e-6)
    # the same call with the forward call's workspace handed over (gates and chunk states reused
    # instead of recomputed) must give the same numbers
    out2 = tfla.mlstm_bwd(dev["q"], dev["k"], dev["v"], dev["i_pre"], dev["f_pre"], dev["dH"],
                          fwd["n_out"], fwd["m_out"], dev.get("C0"), dev.get("n0"), dev.get("m0"), dCn,
                          chunk=w.chunk, variant=w.variant, eps=1e-6, fwd_workspace=fwd["workspace"])
    torch.cuda.synchronize()
    for k_ in ("dq", "dk", "dv", "d_i_pre", "d_f_pre", "dC0"):
        a_, b_ = out[k_].float(), out2[k_].float()
        assert float((a_ - b_).abs().max()) <= 1e-6 * float(a_.abs().max()), k_
    oi = gu.oracle_inputs(d)
    ref = orc.chunkwise_bwd(**oi, dH=gu.flat(d["dH"]), dCn=None if dCn_np is None else gu.flat(dCn_np),
                            variant=w.variant, eps=1e-6, chunk=oracle_chunk or w.chunk)
    names = dict(dq="dq", dk="dk", dv="dv", d_i_pre="di", d_f_pre="df", dC0="dC0")
    errs = {k_: gu.rel_err(out[k_], ref[r_]) for k_, r_ in names.items()}
    print(w.name, "variant", w.variant, "dtype", w.dtype, w.T, w.dqk, w.dhv, w.chunk, errs, flush=True)
    tol = gu.TOL[w.dtype]
    for k_, e in errs.items():
        assert e <= tol, (k_, e, errs)
    return errs


@pytest.mark.parametrize("variant", [wl.EXP, wl.SIG])
@pytest.mark.parametrize("dtype", [wl.BF16, wl.F32])
@pytest.mark.parametrize("shape", [(256, 64, 64, 64), (512, 64, 128, 128), (512, 128, 64, 256), (384, 128, 128, 192)])
def test_bwd_small(variant, dtype, shape):
    T, dqk, dhv, chunk = shape
    run_case(wl.small(variant, dtype, B=1, NH=2, T=T, dqk=dqk, dhv=dhv, chunk=chunk, seed=31 + T + dqk),
             with_dCn=(T == 512), oracle_chunk=96 if T == 384 else None)


@pytest.mark.parametrize("variant", [wl.EXP, wl.SIG])
def test_bwd_7b_head_shape_bf16(variant):
    run_case(wl.small(variant, wl.BF16, B=1, NH=1, T=1024, dqk=256, dhv=512, chunk=256, seed=41), with_dCn=True)


@pytest.mark.parametrize("variant", [wl.EXP, wl.SIG])
@pytest.mark.parametrize("chunk", [64, 192])
def test_bwd_wide_heads_with_chunks_that_are_not_multiples_of_128(variant, chunk):
    # the 512-wide contraction of dQ / dK with the two-wavefront workgroups (their block width differs from
    # the four-wavefront case, and the row-dot buffers are sized from it)
    run_case(wl.small(variant, wl.BF16, B=1, NH=2, T=384, dqk=256, dhv=512, chunk=chunk, seed=43 + chunk), with_dCn=True)


@pytest.mark.parametrize("variant", [wl.EXP, wl.SIG])
@pytest.mark.parametrize("dqk,dhv", [(1024, 1024), (256, 1024), (1024, 128)])
def test_bwd_head_dimensions_above_512_with_upstream_state_gradient(variant, dqk, dhv):
    # contractions over 1024 columns run as two 512-wide launches; dC_T given, so <C_T, dC_T> and dC_0 are covered
    run_case(wl.small(variant, wl.BF16, B=1, NH=1, T=512, dqk=dqk, dhv=dhv, chunk=128, seed=45 + dqk // 64 + dhv), with_dCn=True)


@pytest.mark.parametrize("variant", [wl.EXP, wl.SIG])
@pytest.mark.parametrize("T,dqk,dhv,chunk", [(16384, 64, 128, 128), (9000, 64, 64, 64), (12288, 128, 64, 2048)])
def test_bwd_long_sequences_take_the_anchored_gate_scan(variant, T, dqk, dhv, chunk):
    # the forget-gate gradient scan is anchored with <C_k, dC_k> every few chunks: its error must not grow with T
    # (blocks of four chunks, of one chunk at L = 2048, and a last block that is not full at T = 9000)
    run_case(wl.small(variant, wl.BF16, B=1, NH=2, T=T, dqk=dqk, dhv=dhv, chunk=chunk, seed=47 + chunk), with_dCn=True,
             oracle_chunk=256)
