"""Pins for the layer-level oracle (soft-cap, NORM, output gate, transfer gains).  CPU only.

L1  soft-cap: bounded by c, odd, identity for small arguments (first terms of the series),
    switched off by c = 0; derivative against central differences
L2  NORM against the library routines of PyTorch (independent implementations of the textbook
    RMS norm / LayerNorm), and the invariants of the definition (unit RMS; zero mean, unit variance)
L3  NORM + output gate backward against central finite differences of the forward
L4  whole layer backward (soft-cap -> cell -> NORM -> gate): mLSTMsig against finite differences
    of the layer forward (exact gradient there), mLSTMexp against the frozen-normaliser chain
L5  transfer gains: what Sec. 4.1 states about Fig. "transfer behavior": the gain after the norm
    passes (about 1) or suppresses (about 0) depending on the input gate, mLSTMsig behaves like
    mLSTMexp, and a larger norm epsilon moves the transition towards larger input gate values
"""
import math

import numpy as np
import pytest
import torch

from oracle import layer_oracle as lo
from oracle import mlstm_oracle as orc

EXP, SIG = orc.EXP, orc.SIG


# ---------------------------------------------------------------- L1
def test_l1_softcap_properties():
    x = np.linspace(-80.0, 80.0, 4001)
    y = lo.softcap(x, 15.0)
    assert np.all(np.abs(y) < 15.0) and np.all(np.diff(y) > 0)
    assert np.allclose(lo.softcap(-x, 15.0), -y, atol=0, rtol=0)
    xs = np.linspace(-0.5, 0.5, 101)
    assert np.max(np.abs(lo.softcap(xs, 15.0) - (xs - xs ** 3 / (3 * 15.0 ** 2) + 2 * xs ** 5 / (15 * 15.0 ** 4)))) < 1e-10   # tanh z = z - z^3/3 + 2 z^5/15 - ...
    assert np.array_equal(lo.softcap(x, 0.0), x)
    assert abs(lo.softcap(1e9, 15.0) - 15.0) < 1e-12
    h = 1e-5
    fd = (lo.softcap(x + h, 15.0) - lo.softcap(x - h, 15.0)) / (2 * h)
    assert np.max(np.abs(fd - lo.softcap_grad(x, 15.0))) < 1e-9


# ---------------------------------------------------------------- L2
@pytest.mark.parametrize("kind", [lo.RMS, lo.LAYER])
def test_l2_norm_matches_library(kind):
    g = np.random.default_rng(5)
    B, NH, T, d = 2, 3, 7, 16
    x = g.standard_normal((B, NH, T, d)) * 3 + 0.7
    gamma = g.standard_normal((NH, d)); beta = g.standard_normal((NH, d))
    y = lo.norm_fwd(x, gamma, beta, kind, 1e-6)
    xt = torch.from_numpy(x)
    for h in range(NH):
        if kind == lo.RMS:
            ref = torch.nn.functional.rms_norm(xt[:, h], (d,), torch.from_numpy(gamma[h]), 1e-6)
        else:
            ref = torch.nn.functional.layer_norm(xt[:, h], (d,), torch.from_numpy(gamma[h]), torch.from_numpy(beta[h]), 1e-6)
        assert np.max(np.abs(y[:, h] - ref.numpy())) < 1e-12


def test_l2_norm_invariants():
    g = np.random.default_rng(6)
    x = g.standard_normal((1, 2, 5, 64)) * 10 + 3
    y = lo.norm_fwd(x, None, None, lo.RMS, 0.0)
    assert np.allclose((y * y).mean(-1), 1.0, atol=1e-12)
    assert np.allclose(lo.norm_fwd(7.0 * x, None, None, lo.RMS, 0.0), y, atol=1e-12)      # scale invariance
    z = lo.norm_fwd(x, None, None, lo.LAYER, 0.0)
    assert np.allclose(z.mean(-1), 0.0, atol=1e-12) and np.allclose(z.var(-1), 1.0, atol=1e-12)
    # an epsilon far above mean(x^2) turns the RMS norm into a plain scaling by 1/sqrt(eps)
    big = lo.norm_fwd(1e-6 * x, None, None, lo.RMS, 1.0)
    assert np.allclose(big, 1e-6 * x, rtol=1e-9)
    # for inputs with zero mean both norms agree (App. D.2, experiment setup)
    xc = x - x.mean(-1, keepdims=True)
    assert np.allclose(lo.norm_fwd(xc, None, None, lo.RMS, 1e-6), lo.norm_fwd(xc, None, None, lo.LAYER, 1e-6), atol=1e-12)


# ---------------------------------------------------------------- L3
def _fd(fun, x, dy, h=1e-6):
    """central differences of sum(dy * fun(x)) with respect to every entry of x"""
    gnum = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        idx = it.multi_index
        old = x[idx]
        x[idx] = old + h; fp = (dy * fun()).sum()
        x[idx] = old - h; fm = (dy * fun()).sum()
        x[idx] = old
        gnum[idx] = (fp - fm) / (2 * h)
    return gnum


@pytest.mark.parametrize("kind", [lo.RMS, lo.LAYER])
@pytest.mark.parametrize("gate", [False, True])
def test_l3_norm_gate_backward_finite_differences(kind, gate):
    g = np.random.default_rng(7)
    B, NH, T, d = 2, 2, 3, 6
    h = g.standard_normal((B, NH, T, d)) + 0.3
    o = g.standard_normal((B, NH, T, d)) if gate else None
    gamma = 1 + 0.3 * g.standard_normal((NH, d)); beta = 0.2 * g.standard_normal((NH, d))
    dy = g.standard_normal((B, NH, T, d))
    fun = lambda: lo.norm_gate_fwd(h, o, gamma, beta, kind, 1e-3)
    r = lo.norm_gate_bwd(h, dy, o, gamma, beta, kind, 1e-3)
    assert np.max(np.abs(_fd(fun, h, dy) - r["dh"])) < 1e-7
    assert np.max(np.abs(_fd(fun, gamma, dy) - r["dgamma"])) < 1e-7
    if gate:
        assert np.max(np.abs(_fd(fun, o, dy) - r["do_pre"])) < 1e-7
    else:
        assert r["do_pre"] is None
    if kind == lo.LAYER:
        assert np.max(np.abs(_fd(fun, beta, dy) - r["dbeta"])) < 1e-7
    else:
        assert r["dbeta"] is None


# ---------------------------------------------------------------- L4
def _layer_case(seed, B=1, NH=2, T=10, dqk=4, dhv=6):
    g = np.random.default_rng(seed)
    return dict(q=g.standard_normal((B, NH, T, dqk)), k=g.standard_normal((B, NH, T, dqk)),
                v=g.standard_normal((B, NH, T, dhv)), i_pre=4 * g.standard_normal((B, NH, T)),
                f_pre=4 * g.standard_normal((B, NH, T)) + 2, o_pre=g.standard_normal((B, NH, T, dhv)),
                gamma=1 + 0.2 * g.standard_normal((NH, dhv)), beta=0.1 * g.standard_normal((NH, dhv)))


@pytest.mark.parametrize("kind", [lo.RMS, lo.LAYER])
def test_l4_layer_backward_sig_is_exact(kind):
    d = _layer_case(11)
    g = np.random.default_rng(12)
    dy = g.standard_normal(d["o_pre"].shape)
    kw = dict(variant=SIG, gate_softcap=5.0, kind=kind, norm_eps=1e-3)
    fun = lambda: lo.layer_fwd(**d, **kw)["y"]
    r = lo.layer_bwd(**d, dy=dy, chunk=4, **kw)
    for name, key in (("q", "dq"), ("k", "dk"), ("v", "dv"), ("i_pre", "d_i_pre"), ("f_pre", "d_f_pre"),
                      ("o_pre", "do_pre"), ("gamma", "dgamma")):
        num = _fd(fun, d[name], dy)
        assert np.max(np.abs(num - r[key])) < 2e-7 * max(1.0, np.max(np.abs(num))), name


def test_l4_layer_backward_exp_chain():
    # mLSTMexp: the cell's backward holds the normaliser constant (App. B.3), so the layer gradient is
    # that backward applied to the exact gradient of NORM + gate, times the soft-cap derivative
    d = _layer_case(13)
    g = np.random.default_rng(14)
    dy = g.standard_normal(d["o_pre"].shape)
    kw = dict(variant=EXP, gate_softcap=15.0, kind=lo.RMS, norm_eps=1e-6, eps=1e-6)
    r = lo.layer_bwd(**d, dy=dy, chunk=5, **kw)
    f = lo.layer_fwd(**d, **kw)
    ng = lo.norm_gate_bwd(f["H"], dy, d["o_pre"], d["gamma"], d["beta"], lo.RMS, 1e-6)
    B, NH = d["q"].shape[:2]
    sl = lambda a: a.reshape((-1,) + a.shape[2:])
    ref = orc.quadratic_bwd(sl(d["q"]), sl(d["k"]), sl(d["v"]), sl(lo.softcap(d["i_pre"], 15.0)),
                            sl(lo.softcap(d["f_pre"], 15.0)), sl(ng["dh"]), variant=EXP, eps=1e-6)
    assert np.max(np.abs(sl(r["dq"]) - ref["dq"])) < 1e-10
    assert np.max(np.abs(sl(r["d_i_pre"]) - ref["di"] * sl(lo.softcap_grad(d["i_pre"], 15.0)))) < 1e-10
    assert np.max(np.abs(sl(r["d_f_pre"]) - ref["df"] * sl(lo.softcap_grad(d["f_pre"], 15.0)))) < 1e-10
    # the soft-cap is what the cell sees: capping by hand and switching it off gives the same output
    d2 = dict(d, i_pre=lo.softcap(d["i_pre"], 15.0), f_pre=lo.softcap(d["f_pre"], 15.0))
    assert np.max(np.abs(lo.layer_fwd(**d2, **dict(kw, gate_softcap=0.0))["y"] - f["y"])) < 1e-12


# ---------------------------------------------------------------- L5
def _gains(variant, i_val, f_val, norm_eps=1e-6, T=128, d=32, seed=21):
    g = np.random.default_rng(seed)
    q = g.standard_normal((1, 1, T, d)); k = g.standard_normal((1, 1, T, d)); v = g.standard_normal((1, 1, T, d))
    o = orc.recurrent_fwd(q[0], k[0], v[0], np.full((1, T), float(i_val)), np.full((1, T), float(f_val)),
                          variant=variant, eps=0.0)
    gb, ga = lo.transfer_gain(o["H"][None], v, lo.RMS, norm_eps)
    return float(gb[0, 0]), float(ga[0, 0])


def test_l5_gain_worked_by_hand():
    """Gain equation of Sec. 4.1 on two steps of two columns, worked by hand: the ratio of max-norms is formed at
    every step and then averaged.  h = [[1, -2], [3, 0.5]], v = [[2, 1], [1, -4]]:
      before the norm: (2/2 + 3/4) / 2 = 0.875           (the ratio of the averages would be 2.5/3 = 0.8333)
      RMS norm (eps = 0): rows scale by 1/sqrt(2.5) and 1/sqrt(4.625): maxima 2/sqrt(2.5), 3/sqrt(4.625)
      LayerNorm (eps = 0): both rows become (1, -1): maxima 1, 1 -> (1/2 + 1/4) / 2 = 0.375"""
    h = np.array([[1.0, -2.0], [3.0, 0.5]])[None, None]
    v = np.array([[2.0, 1.0], [1.0, -4.0]])[None, None]
    gb, ga = lo.transfer_gain(h, v, lo.RMS, 0.0)
    assert gb.shape == (1, 1) and abs(gb[0, 0] - 0.875) < 1e-15
    want = 0.5 * (2.0 / math.sqrt(2.5) / 2.0 + 3.0 / math.sqrt(4.625) / 4.0)      # 0.490604...
    assert abs(want - 0.4906) < 1e-4 and abs(ga[0, 0] - want) < 1e-14
    gb, ga = lo.transfer_gain(h, v, lo.LAYER, 0.0)
    assert abs(gb[0, 0] - 0.875) < 1e-15 and abs(ga[0, 0] - 0.375) < 1e-14
    # two (batch, head) slices are averaged separately
    h2 = np.concatenate([h, 2.0 * h], axis=1)
    v2 = np.concatenate([v, v], axis=1)
    gb, _ = lo.transfer_gain(h2, v2, lo.RMS, 0.0)
    assert gb.shape == (1, 2) and abs(gb[0, 1] - 1.75) < 1e-15


@pytest.mark.parametrize("variant", [EXP, SIG])
def test_l5_gain_passes_and_suppresses(variant):
    # open input gate: the signal passes the norm with a gain of about one
    _, ga = _gains(variant, 4.0, 4.0)
    assert 0.6 < ga < 1.6
    # far closed input gate: suppressed (the norm epsilon dominates the denominator)
    _, ga = _gains(variant, -12.0, 4.0)
    assert ga < 0.05
    # monotone transition in between
    gs = [_gains(variant, iv, 4.0)[1] for iv in (-12, -10, -8, -6, -4, -2, 0)]
    assert all(b >= a - 1e-3 for a, b in zip(gs, gs[1:]))


def test_l5_sig_matches_exp_after_norm():
    for iv in (-10.0, -7.0, -4.0, 0.0, 4.0):
        for fv in (-2.0, 3.0, 8.0):
            ge = _gains(EXP, iv, fv)[1]; gs = _gains(SIG, iv, fv)[1]
            assert abs(ge - gs) < 0.15 * max(ge, gs) + 0.02, (iv, fv, ge, gs)


def test_l5_larger_epsilon_shifts_transition_up():
    # the input gate value at which the gain crosses 1/2 grows with the norm epsilon
    def crossing(eps):
        ivs = np.arange(-12.0, 4.01, 0.5)
        gs = np.array([_gains(EXP, iv, 4.0, eps)[1] for iv in ivs])
        return ivs[np.argmax(gs > 0.5 * gs[-1])]
    assert crossing(1e-2) > crossing(1e-6) > crossing(1e-8)
