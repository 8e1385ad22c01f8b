"""GPU parity at the full benchmark configurations, in the launch configuration bench.py times.
The kernels run on the whole problem; the fp64 oracle is evaluated on a sample of (batch, head)
slices (drawn from the same per-slice streams, so they are the same numbers) and compared
element by element on those slices."""
import dataclasses

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import mlstm_oracle as orc

pytestmark = pytest.mark.gpu


def _sample(w):
    """(batch, head) slices checked against the oracle: the first, the last, and one from the middle of the
    second batch element (or of the heads when there is one batch element) -- the slices a wrong grid decode,
    slice stride or workspace offset would show in"""
    BH = w.B * w.NH
    mid = (w.NH + w.NH // 2 + 1) if w.B > 1 else w.NH // 2
    return sorted({0, min(mid, BH - 1), BH - 1})


def _run_fwd(w, dev):
    import paper_2503_14376_amd as tfla
    return tfla.mlstm_fwd(dev["q"], dev["k"], dev["v"], dev["i_pre"], dev["f_pre"], dev.get("C0"), dev.get("n0"),
                          dev.get("m0"), chunk=w.chunk, variant=w.variant, eps=1e-6)


def _sub(t, idx):
    """the (batch*head) slices idx of a (B, NH, ...) device tensor, as (1, len(idx), ...)"""
    sel = torch.as_tensor(idx, device=t.device, dtype=torch.long)
    return t.reshape((-1,) + tuple(t.shape[2:])).index_select(0, sel).unsqueeze(0)


def _check_fwd_sample(w, out, ref, idx):
    from tests import gpu_util as gu
    sub = {k_: _sub(v_, idx) for k_, v_ in out.items() if isinstance(v_, torch.Tensor) and v_.dim() >= 2 and k_ != "workspace"}
    errs = gu.check_fwd(w, None, sub, ref)
    print(w.name, "chunk", w.chunk, errs, flush=True)
    return errs


def test_config1_forward_with_initial_state():
    from tests import gpu_util as gu
    w = wl.CONFIGS["c1"]
    d = wl.make_inputs(w)
    out = _run_fwd(w, gu.dev_inputs(w, d))
    idx = _sample(w)
    ds = wl.make_inputs(w, slices=idx)
    ref = orc.recurrent_fwd(**gu.oracle_inputs(ds), variant=w.variant, eps=1e-6)
    _check_fwd_sample(w, out, ref, idx)


def test_config2_sig_chunk_sweep():
    """mLSTMsig at the 7B head shape; the result must not depend on the chunk size."""
    from tests import gpu_util as gu
    w0 = wl.CONFIGS["c2"]
    d = wl.make_inputs(w0)
    dev = gu.dev_inputs(w0, d)
    idx = _sample(w0)
    ds = wl.make_inputs(w0, slices=idx)
    ref = orc.recurrent_fwd(**gu.oracle_inputs(ds), variant=w0.variant, eps=1e-6)
    for L in wl.C2_CHUNKS:
        w = dataclasses.replace(w0, chunk=L)
        out = _run_fwd(w, dev)
        _check_fwd_sample(w, out, ref, idx)
        for key in ("nn", "mn", "n_out", "m_out"):
            assert float(out[key].abs().max()) == 0.0     # no normaliser / max state in mLSTMsig


def test_config3_long_context_final_state_and_continuation():
    from tests import gpu_util as gu
    import paper_2503_14376_amd as tfla
    w = wl.CONFIGS["c3"]
    d = wl.make_inputs(w)
    dev = gu.dev_inputs(w, d)
    out = _run_fwd(w, dev)
    idx = _sample(w)
    ds = wl.make_inputs(w, slices=idx)
    ref = orc.recurrent_fwd(**gu.oracle_inputs(ds), variant=w.variant, eps=1e-6)
    _check_fwd_sample(w, out, ref, idx)
    # chunked continuation: two calls over the halves, the state handed across, equal one call
    T1 = w.T // 2
    a = {k_: v_[:, :, :T1].contiguous() for k_, v_ in dev.items()}
    b = {k_: v_[:, :, T1:].contiguous() for k_, v_ in dev.items()}
    oa = tfla.mlstm_fwd(a["q"], a["k"], a["v"], a["i_pre"], a["f_pre"], chunk=w.chunk, variant=w.variant, eps=1e-6)
    ob = tfla.mlstm_fwd(b["q"], b["k"], b["v"], b["i_pre"], b["f_pre"], oa["Cn"], oa["nn"], oa["mn"], chunk=w.chunk,
                        variant=w.variant, eps=1e-6)
    H2 = torch.cat([oa["H"], ob["H"]], dim=2).float()
    H1 = out["H"].float()
    assert float((H2 - H1).abs().max() / H1.abs().max()) <= 2e-2
    assert float((ob["Cn"] - out["Cn"]).abs().max() / out["Cn"].abs().max()) <= 2e-2
    assert float((ob["mn"] - out["mn"]).abs().max()) <= 1e-3


@pytest.mark.parametrize("name", ["c4", "c4sig"])
def test_config4_forward_backward(name):
    from tests import gpu_util as gu
    import paper_2503_14376_amd as tfla
    w = wl.CONFIGS[name]
    d = wl.make_inputs(w)
    dev = gu.dev_inputs(w, d)
    fwd = _run_fwd(w, dev)
    bwd = tfla.mlstm_bwd(dev["q"], dev["k"], dev["v"], dev["i_pre"], dev["f_pre"], dev["dH"], fwd["n_out"], fwd["m_out"],
                         chunk=w.chunk, variant=w.variant, eps=1e-6, fwd_workspace=fwd["workspace"])
    torch.cuda.synchronize()
    idx = _sample(w)
    ds = wl.make_inputs(w, slices=idx)
    oi = gu.oracle_inputs(ds)
    ref_f = orc.recurrent_fwd(**oi, variant=w.variant, eps=1e-6)
    _check_fwd_sample(w, fwd, ref_f, idx)
    ref = orc.chunkwise_bwd(**oi, dH=gu.flat(ds["dH"]), variant=w.variant, eps=1e-6, chunk=w.chunk)
    names = dict(dq="dq", dk="dk", dv="dv", d_i_pre="di", d_f_pre="df", dC0="dC0")
    errs = {k_: gu.rel_err(_sub(bwd[k_], idx), ref[r_]) for k_, r_ in names.items()}
    print(w.name, "backward", errs, flush=True)
    for k_, e in errs.items():
        assert e <= 2e-2, (k_, e, errs)
