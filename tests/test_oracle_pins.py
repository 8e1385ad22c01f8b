"""Pins for the fp64 oracle: what the paper and the mathematics fix, checked without
any reference implementation.  CPU only.

P1  recurrence (Sec. 2.1 / 4.1)  ==  fully parallel form (App. B.1) on tiny inputs
P2  chunkwise form (App. B.2) is invariant to the chunk size, L=1..T
P3  the max state cancels (App. D.1): direct evaluation of the unstabilised cell;
    gauge invariance of the initial state
P4  special cases that reduce to textbook formulas
P5  continuation across a split of the sequence
P6  backward: central finite differences of the frozen-normaliser objective;
    chunkwise backward (App. B.3) == definition, for several L
P7  the count model reproduces the numbers the paper prints
P8  gate pre-activations up to |x| = 300: every forward form and both backward definitions against the
    unstabilised cell in 150-digit arithmetic
"""
import math
import os

import numpy as np
import pytest

from oracle import count_model as cm
from oracle import mlstm_oracle as orc

EXP, SIG = orc.EXP, orc.SIG


def rand_case(seed, S=2, T=12, dqk=4, dhv=5, f_mean=1.0, state=True):
    g = np.random.default_rng(seed)
    d = dict(q=g.standard_normal((S, T, dqk)), k=g.standard_normal((S, T, dqk)),
             v=g.standard_normal((S, T, dhv)), i_pre=g.standard_normal((S, T)),
             f_pre=g.standard_normal((S, T)) + f_mean)
    if state:
        d.update(C0=0.3 * g.standard_normal((S, dqk, dhv)), n0=0.3 * g.standard_normal((S, dqk)),
                 m0=0.5 * g.standard_normal((S,)))
    else:
        d.update(C0=None, n0=None, m0=None)
    return d


def close(a, b, tol=1e-11):
    scale = max(1.0, float(np.max(np.abs(b))))
    assert np.max(np.abs(a - b)) <= tol * scale, (np.max(np.abs(a - b)), scale)


# ---------------------------------------------------------------- P1
@pytest.mark.parametrize("variant", [EXP, SIG])
@pytest.mark.parametrize("state", [False, True])
def test_p1_recurrent_equals_quadratic(variant, state):
    d = rand_case(1, T=40, dqk=6, dhv=7, state=state)
    r = orc.recurrent_fwd(**d, variant=variant, eps=1e-6)
    p = orc.quadratic_fwd(**d, variant=variant, eps=1e-6)
    close(r["H"], p["H"])
    close(r["n_out"], p["n_out"])
    close(r["m_out"], p["m_out"])


def test_p1_paper_parallel_form_without_m0():
    # App. B.1 as printed has no initial state and takes the row max over D~ only
    # (m0 = -inf); H must not depend on that choice (the max state cancels).
    d = rand_case(2, T=24, state=False)
    r = orc.recurrent_fwd(**d, variant=EXP)
    S, T, dqk = d["q"].shape
    for s in range(S):
        fbar = orc.log_sigmoid(d["f_pre"][s]); cum = np.cumsum(fbar)
        Dt = cum[:, None] - cum[None, :] + d["i_pre"][s][None, :]
        Dt[np.triu_indices(T, 1)] = -np.inf
        m = Dt.max(axis=1)
        Sbar = (d["q"][s] @ d["k"][s].T) / math.sqrt(dqk) * np.exp(Dt - m[:, None])
        n = np.maximum(np.abs(Sbar.sum(1)), np.exp(-m))
        close(r["H"][s], (Sbar / n[:, None]) @ d["v"][s])


# ---------------------------------------------------------------- P2
@pytest.mark.parametrize("variant", [EXP, SIG])
def test_p2_chunk_size_invariance_forward(variant):
    d = rand_case(3, T=30, dqk=5, dhv=6)
    r = orc.recurrent_fwd(**d, variant=variant, eps=1e-6)
    for L in (1, 2, 3, 5, 7, 8, 15, 29, 30, 64):
        c = orc.chunkwise_fwd(**d, variant=variant, eps=1e-6, chunk=L)
        for key in ("H", "Cn", "nn", "mn", "n_out", "m_out"):
            close(c[key], r[key])


def test_p2_stable_and_unstable_a_agree():
    # App. B.2's listing: a_k formed by a shifted reverse cumsum vs. g - b + i-bar
    g = np.random.default_rng(4)
    f = g.standard_normal(64) + 3; i = g.standard_normal(64)
    gk, b, a, ibar = orc.chunk_gates(i, f, EXP)
    close(a, gk - b + ibar, 1e-13)
    assert a[-1] == ibar[-1] and abs(b[-1] - gk) == 0


# ---------------------------------------------------------------- P3
def unstabilised(d, variant, s):
    """Direct evaluation of the cell without max state (App. D.1, first equation):
    C_t = sigma(f~) C_{t-1} + exp(i~) k v^T (resp. sigma(i~)), n_t likewise,
    h = C_t^T q~ / max(|n_t^T q~|, 1).  Returns (H, list of true numerators, C_T true)."""
    q, k, v = d["q"][s], d["k"][s], d["v"][s]
    T, dqk = q.shape
    m0 = 0.0 if (d["m0"] is None or variant == SIG) else d["m0"][s]
    C = np.zeros((dqk, v.shape[1])) if d["C0"] is None else d["C0"][s] * math.exp(m0)
    n = np.zeros(dqk) if d["n0"] is None else d["n0"][s] * math.exp(m0)
    H = np.zeros_like(v); nums = []
    for t in range(T):
        fg = 1 / (1 + math.exp(-d["f_pre"][s, t]))
        ig = math.exp(d["i_pre"][s, t]) if variant == EXP else 1 / (1 + math.exp(-d["i_pre"][s, t]))
        C = fg * C + ig * np.outer(k[t], v[t]); n = fg * n + ig * k[t]
        qs = q[t] / math.sqrt(dqk)
        num = C.T @ qs; nums.append(num)
        H[t] = num / (max(abs(n @ qs), 1.0) if variant == EXP else 1.0)
    return H, np.array(nums), C


@pytest.mark.parametrize("variant", [EXP, SIG])
def test_p3_max_state_cancels(variant):
    d = rand_case(5, T=25)
    r = orc.recurrent_fwd(**d, variant=variant, eps=0.0)
    for s in range(d["q"].shape[0]):
        H, _, Ctrue = unstabilised(d, variant, s)
        close(r["H"][s], H, 1e-10)
        close(r["Cn"][s] * math.exp(r["mn"][s]), Ctrue, 1e-10)


def test_p3_gauge_invariance():
    d = rand_case(6, T=20)
    r0 = orc.recurrent_fwd(**d, variant=EXP)
    c = 1.7
    d2 = dict(d, C0=d["C0"] * math.exp(-c), n0=d["n0"] * math.exp(-c), m0=d["m0"] + c)
    r1 = orc.recurrent_fwd(**d2, variant=EXP)
    close(r0["H"], r1["H"], 1e-10)


# ---------------------------------------------------------------- P4
def test_p4_sig_saturated_gates_is_causal_linear_attention():
    d = rand_case(7, T=16, state=False)
    d["i_pre"][:] = 40.0; d["f_pre"][:] = 40.0
    r = orc.recurrent_fwd(**d, variant=SIG)
    for s in range(2):
        A = np.tril(d["q"][s] @ d["k"][s].T) / math.sqrt(d["q"].shape[-1])
        close(r["H"][s], A @ d["v"][s], 1e-10)


def test_p4_exp_unit_gates_is_normalised_linear_attention():
    d = rand_case(8, T=16, state=False)
    d["i_pre"][:] = 0.0; d["f_pre"][:] = 40.0
    r = orc.recurrent_fwd(**d, variant=EXP)
    for s in range(2):
        A = np.tril(d["q"][s] @ d["k"][s].T) / math.sqrt(d["q"].shape[-1])
        den = np.maximum(np.abs(A.sum(1)), 1.0)
        close(r["H"][s], (A @ d["v"][s]) / den[:, None], 1e-10)


@pytest.mark.parametrize("variant", [EXP, SIG])
def test_p4_forget_everything_depends_on_current_step_only(variant):
    # f~ = -40: sigma(f~) ~ 4e-18, the state is reset at every step (document boundary)
    d = rand_case(9, T=10, state=True)
    d["f_pre"][:] = -40.0
    r = orc.recurrent_fwd(**d, variant=variant)
    for s in range(2):
        for t in range(10):
            stt = d["q"][s, t] @ d["k"][s, t] / math.sqrt(d["q"].shape[-1])
            it = d["i_pre"][s, t]
            if variant == EXP:
                ref = stt * d["v"][s, t] / max(abs(stt), math.exp(-it))   # m_t = i~_t
                assert abs(r["m_out"][s, t] - it) < 1e-9
            else:
                ref = stt * d["v"][s, t] / (1 + math.exp(-it))
            close(r["H"][s, t], ref, 1e-9)


def test_p4_single_step_by_hand():
    q = np.array([[[2.0, 0.0]]]); k = np.array([[[1.0, 1.0]]]); v = np.array([[[3.0, -1.0, 0.5]]])
    i_pre = np.array([[0.5]]); f_pre = np.array([[0.0]])
    r = orc.recurrent_fwd(q, k, v, i_pre, f_pre, variant=EXP)
    # m_1 = max(log(1/2) + 0, 0.5) = 0.5; i = exp(0) = 1; C = k v^T; n = k; q~ = q/sqrt(2)
    s = 2.0 / math.sqrt(2.0)
    den = max(abs(s), math.exp(-0.5))
    close(r["H"][0, 0], s * v[0, 0] / den, 1e-14)
    assert r["mn"][0] == 0.5
    r = orc.recurrent_fwd(q, k, v, i_pre, f_pre, variant=SIG)
    close(r["H"][0, 0], s * v[0, 0] / (1 + math.exp(-0.5)), 1e-14)


# ---------------------------------------------------------------- P5
@pytest.mark.parametrize("variant", [EXP, SIG])
def test_p5_continuation(variant):
    d = rand_case(10, T=33)
    full = orc.recurrent_fwd(**d, variant=variant, eps=1e-6)
    T1 = 14
    a = {k_: (v_[:, :T1] if k_ in ("q", "k", "v", "i_pre", "f_pre") else v_) for k_, v_ in d.items()}
    ra = orc.recurrent_fwd(**a, variant=variant, eps=1e-6)
    b = {k_: v_[:, T1:] for k_, v_ in d.items() if k_ in ("q", "k", "v", "i_pre", "f_pre")}
    rb = orc.recurrent_fwd(**b, C0=ra["Cn"], n0=ra["nn"], m0=ra["mn"], variant=variant, eps=1e-6)
    close(np.concatenate([ra["H"], rb["H"]], axis=1), full["H"])
    close(rb["Cn"], full["Cn"]); close(rb["nn"], full["nn"]); close(rb["mn"], full["mn"])


# ---------------------------------------------------------------- P6
def frozen_objective(d, dH, dCn, variant, consts):
    """l(x) = sum_t <dH_t, Num_t(x)> c_t + <dCn, C_T(x)> c_T with the unstabilised numerators
    and constants c_t = 1/(den_t e^{m_t}), c_T = e^{-m_T} frozen at the base point."""
    tot = 0.0
    for s in range(d["q"].shape[0]):
        _, nums, Ctrue = unstabilised(d, variant, s)
        tot += np.sum(dH[s] * nums * consts["c"][s][:, None])
        if dCn is not None:
            tot += np.sum(dCn[s] * Ctrue) * consts["cT"][s]
    return tot


@pytest.mark.parametrize("variant", [EXP, SIG])
@pytest.mark.parametrize("with_dCn", [False, True])
def test_p6_backward_matches_finite_differences(variant, with_dCn):
    d = rand_case(11, S=1, T=9, dqk=3, dhv=4)
    g = np.random.default_rng(12)
    dH = g.standard_normal(d["v"].shape)
    dCn = g.standard_normal(d["C0"].shape) if with_dCn else None
    eps = 1e-6 if variant == EXP else 0.0
    f = orc.recurrent_fwd(**d, variant=variant, eps=eps)
    if variant == EXP:
        den = np.maximum(np.abs(f["n_out"]), np.exp(-f["m_out"])) + eps
        consts = dict(c=1.0 / (den * np.exp(f["m_out"])), cT=np.exp(-f["mn"]))
    else:
        consts = dict(c=np.ones_like(f["n_out"]), cT=np.ones(1))
    grads = orc.quadratic_bwd(**d, dH=dH, dCn=dCn, variant=variant, eps=eps)
    names = dict(q="dq", k="dk", v="dv", i_pre="di", f_pre="df", C0="dC0")
    h = 1e-5
    for key, gname in names.items():
        x = d[key]
        fd = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            xp = x.copy(); xp[idx] += h
            xm = x.copy(); xm[idx] -= h
            fd[idx] = (frozen_objective(dict(d, **{key: xp}), dH, dCn, variant, consts)
                       - frozen_objective(dict(d, **{key: xm}), dH, dCn, variant, consts)) / (2 * h)
        err = np.max(np.abs(fd - grads[gname])) / max(1e-30, np.max(np.abs(fd)))
        assert err < 2e-7, (key, err)


def test_p6_sig_backward_is_the_true_gradient():
    # no normaliser in mLSTMsig: the definition is the plain gradient of sum <dH, H>
    d = rand_case(13, S=1, T=8, dqk=3, dhv=3)
    g = np.random.default_rng(14)
    dH = g.standard_normal(d["v"].shape)
    grads = orc.quadratic_bwd(**d, dH=dH, variant=SIG)
    h = 1e-5
    for key, gname in dict(q="dq", f_pre="df", i_pre="di", C0="dC0").items():
        x = d[key]; fd = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            xp = x.copy(); xp[idx] += h
            xm = x.copy(); xm[idx] -= h
            lp = np.sum(dH * orc.recurrent_fwd(**dict(d, **{key: xp}), variant=SIG)["H"])
            lm = np.sum(dH * orc.recurrent_fwd(**dict(d, **{key: xm}), variant=SIG)["H"])
            fd[idx] = (lp - lm) / (2 * h)
        assert np.max(np.abs(fd - grads[gname])) / np.max(np.abs(fd)) < 2e-7, key


@pytest.mark.parametrize("variant", [EXP, SIG])
@pytest.mark.parametrize("with_dCn", [False, True])
def test_p6_chunkwise_backward_equals_definition(variant, with_dCn):
    d = rand_case(15, S=2, T=24, dqk=4, dhv=5)
    g = np.random.default_rng(16)
    dH = g.standard_normal(d["v"].shape)
    dCn = g.standard_normal(d["C0"].shape) if with_dCn else None
    ref = orc.quadratic_bwd(**d, dH=dH, dCn=dCn, variant=variant, eps=1e-6)
    for L in (1, 2, 3, 4, 6, 7, 12, 24):
        c = orc.chunkwise_bwd(**d, dH=dH, dCn=dCn, variant=variant, eps=1e-6, chunk=L)
        for key in ref:
            close(c[key], ref[key], 1e-10)


def test_p6_gate_gradient_identity():
    # sum over the log-weights: q.dq and k.dk are the row / column sums of the log-weight
    # gradients, so  d f-bar_s = sum_{t>=s} (q_t.dq_t - k_t.dk_t) + <C_T, dC_T>.
    d = rand_case(17, S=1, T=20, dqk=4, dhv=5)
    g = np.random.default_rng(18)
    dH = g.standard_normal(d["v"].shape); dCn = g.standard_normal(d["C0"].shape)
    r = orc.quadratic_bwd(**d, dH=dH, dCn=dCn, variant=EXP, eps=1e-6)
    f = orc.recurrent_fwd(**d, variant=EXP, eps=1e-6)
    R = np.einsum("std,std->st", d["q"], r["dq"]); Cc = np.einsum("std,std->st", d["k"], r["dk"])
    dfbar = np.cumsum((R - Cc)[:, ::-1], axis=1)[:, ::-1] + np.sum(f["Cn"] * dCn)
    close(dfbar * orc.sigmoid(-d["f_pre"]), r["df"], 1e-10)
    close(Cc, r["di"], 1e-10)


# ---------------------------------------------------------------- P7
def golden():
    path = os.path.join(os.path.dirname(__file__), "golden", "count_model_paper_values.txt")
    out = {}
    for line in open(path):
        line = line.split("#")[0].split()
        if len(line) == 2:
            out[line[0]] = float(line[1])
    return out


def test_p7_count_model_reproduces_printed_numbers():
    gold = golden()
    specs = dict(V100=(120e12, 0.9e12), A100=(312e12, 1.935e12), H100=(989e12, 3.35e12), B200=(2250e12, 7.7e12))
    for name, (fl, bw) in specs.items():
        assert round(fl / bw) == gold["accelerator_intensity_" + name]
    # "L=16 for d_hv=512": F_causal between 0.5 and the 0.66 the text suggests for blocked masks
    lo, hi = cm.l_opt_flop(512, 0.5, 0.66), cm.l_opt_flop(512, 0.5, 0.5)
    assert lo <= gold["l_opt_flop_dhv512"] + 0.5 and hi >= gold["l_opt_flop_dhv512"]
    for L in (64, 256):
        for T in (8192,):
            e64 = cm.flops_chunkwise_exp(T, L, 64, 64) / cm.flops_chunkwise_sig(T, L, 64, 64) - 1
            e512 = cm.flops_chunkwise_exp(T, L, 512, 512) / cm.flops_chunkwise_sig(T, L, 512, 512) - 1
            # the text rounds: the chunkwise count gives 1.8 % (L=256) to 2.05 % (L=64)
            assert 0 < e64 < gold["flop_excess_exp_over_sig_d64_max"] * 1.05
            # "about 0.2 %": the chunkwise count gives 0.22 % (L=1024) to 0.33 % (L=16)
            assert 0.5 * gold["flop_excess_exp_over_sig_d512"] < e512 < 2 * gold["flop_excess_exp_over_sig_d512"]
    e = cm.flops_recurrent_exp(1, 512, 512) / cm.flops_recurrent_sig(1, 512, 512) - 1
    assert abs(e - 0.002) < 1e-3
    e = cm.flops_recurrent_exp(1, 64, 64) / cm.flops_recurrent_sig(1, 64, 64) - 1
    assert 0 < e < gold["flop_excess_exp_over_sig_d64_max"]
    e = cm.flops_parallel_exp(8192, 64, 64) / cm.flops_parallel_sig(8192, 64, 64) - 1
    assert 0 < e < gold["flop_excess_exp_over_sig_d64_max"]


def test_p7_count_model_self_consistency():
    T, dhv, p = 8192, 512, 0.5
    dqk = int(dhv * p)
    for L in (64, 256, 1024):
        I = cm.flops_chunkwise_sig(T, L, dqk, dhv) / cm.bytes_chunkwise_sig(T, L, dqk, dhv)
        assert abs(I / cm.intensity_sig_closed_form(L, dhv, p) - 1) < 1e-12
    # closed-form optimum = numerical argmin of the count
    Ls = np.arange(4, 200, 0.01)
    assert abs(Ls[np.argmin(cm.flops_chunkwise_sig(T, Ls, dqk, dhv))] - cm.l_opt_flop(dhv, p)) < 0.02
    a_f, a_b = 989e12, 3.35e12
    tau = cm.flops_chunkwise_sig(T, Ls * 10, dqk, dhv) / a_f + cm.bytes_chunkwise_sig(T, Ls * 10, dqk, dhv) / a_b
    assert abs(Ls[np.argmin(tau)] * 10 - cm.l_opt_runtime(dhv, p, a_f / a_b)) < 0.5
    # L=1 and L=T limits move between the recurrent and the parallel counts (App. G.5, item 2)
    assert cm.flops_chunkwise_sig(T, 1, dqk, dhv) / cm.flops_recurrent_sig(T, dqk, dhv) < 1.01


def _memop_table():
    """rows[(row, column)] = list of (byte_type, c_dqk, c_dhv, c_dqkdhv, c_one) from the golden file."""
    rows = {}
    path = os.path.join(os.path.dirname(__file__), "golden", "recurrent_step_memory_operations.txt")
    for line in open(path):
        line = line.split("#")[0].split()
        if len(line) == 7:
            rows.setdefault((line[0], line[1]), []).append((line[2],) + tuple(int(x) for x in line[3:]))
    return rows


def _memop_eval(entries, dqk, dhv, nbytes):
    return sum(nbytes[t] * (a * dqk + b * dhv + c * dqk * dhv + e) for t, a, b, c, e in entries)


def test_p7_recurrent_step_memory_operations():
    """App. F.2, memory-operation table of the recurrent formulation: the count model equals the sum of the
    table's load and store rows, typed entry by entry into tests/golden/ (not the same expression retyped).
    The printed total row carries the two columns exchanged: it matches load + store of the other column."""
    from oracle import count_model as cm
    tab = _memop_table()
    assert len(tab) == 6
    fn = {"mLSTMexp": cm.bytes_recurrent_step_exp, "mLSTMsig": cm.bytes_recurrent_step_sig}
    other = {"mLSTMexp": "mLSTMsig", "mLSTMsig": "mLSTMexp"}
    for dqk, dhv in ((64, 64), (256, 512), (40, 24)):
        for bq, bi, bc in ((2, 2, 4), (2, 4, 4), (4, 4, 4), (1, 3, 8)):
            nb = {"qkv": bq, "if": bi, "Cmn": bc}
            for col in fn:
                rows_sum = _memop_eval(tab[("load", col)], dqk, dhv, nb) + _memop_eval(tab[("store", col)], dqk, dhv, nb)
                assert fn[col](dqk, dhv, bq, bi, bc) == rows_sum
                assert _memop_eval(tab[("total", other[col])], dqk, dhv, nb) == rows_sum
                assert _memop_eval(tab[("total", col)], dqk, dhv, nb) != rows_sum
    # at the 7B head shape the matrix memory is > 99 % of the traffic: the step is bound by 2 d_qk d_hv floats
    tot = cm.bytes_recurrent_step_exp(256, 512)
    assert 2 * 256 * 512 * 4 / tot > 0.99


# ---------------------------------------------------------------- P8
def _mp_cell(d, dH, variant, s, digits=150):
    """The unstabilised cell (App. D.1, first equation) and the frozen-normaliser gradients of
    l = sum_t <dH_t, H_t>, written as explicit double sums over (t, j) in arbitrary-precision arithmetic:
    no max state, no log-domain reordering, so that nothing of the oracle's stabilisation is shared.
    Zero initial state.  Returns floats."""
    mp = pytest.importorskip("mpmath")
    mp.mp.dps = digits
    F = mp.mpf
    q, k, v = d["q"][s], d["k"][s], d["v"][s]
    T, dqk = q.shape
    dhv = v.shape[1]
    ip = [F(float(x)) for x in d["i_pre"][s]]
    fp = [F(float(x)) for x in d["f_pre"][s]]
    sig = lambda x: 1 / (1 + mp.exp(-x))
    fg = [sig(x) for x in fp]
    ig = [mp.exp(x) if variant == EXP else sig(x) for x in ip]
    rs = 1 / mp.sqrt(dqk)
    qs = [[F(float(q[t, c])) * rs for c in range(dqk)] for t in range(T)]
    kk = [[F(float(k[t, c])) for c in range(dqk)] for t in range(T)]
    vv = [[F(float(v[t, c])) for c in range(dhv)] for t in range(T)]
    gg = [[F(float(dH[s][t, c])) for c in range(dhv)] for t in range(T)]
    # w[t][j] = ig_j * prod_{j < r <= t} fg_r
    w = [[F(0)] * T for _ in range(T)]
    for t in range(T):
        for j in range(t + 1):
            p = ig[j]
            for r in range(j + 1, t + 1):
                p *= fg[r]
            w[t][j] = p
    dot = lambda a, b: sum(x * y for x, y in zip(a, b))
    H = np.zeros((T, dhv)); den = [F(1)] * T
    for t in range(T):
        num = [sum(w[t][j] * dot(qs[t], kk[j]) * vv[j][c] for j in range(t + 1)) for c in range(dhv)]
        nrm = sum(w[t][j] * dot(qs[t], kk[j]) for j in range(t + 1))
        den[t] = max(abs(nrm), F(1)) if variant == EXP else F(1)
        H[t] = [float(x / den[t]) for x in num]
    dq = np.zeros((T, dqk)); dk = np.zeros((T, dqk)); dv = np.zeros((T, dhv)); di = np.zeros(T); df = np.zeros(T)
    E = [[F(0)] * T for _ in range(T)]              # gradient w.r.t. the log of w[t][j]
    for t in range(T):
        for j in range(t + 1):
            E[t][j] = w[t][j] * dot(qs[t], kk[j]) * dot(gg[t], vv[j]) / den[t]
    for t in range(T):
        for c in range(dqk):
            dq[t, c] = float(rs * sum(w[t][j] * dot(gg[t], vv[j]) / den[t] * kk[j][c] for j in range(t + 1)))
    for j in range(T):
        for c in range(dqk):
            dk[j, c] = float(sum(w[t][j] * dot(gg[t], vv[j]) / den[t] * qs[t][c] for t in range(j, T)))
        for c in range(dhv):
            dv[j, c] = float(sum(w[t][j] * dot(qs[t], kk[j]) * gg[t][c] / den[t] for t in range(j, T)))
        dlog_i = sum(E[t][j] for t in range(j, T))                      # d/d log(ig_j)
        di[j] = float(dlog_i if variant == EXP else dlog_i * sig(-ip[j]))
        dlog_f = sum(E[t][jj] for t in range(j, T) for jj in range(j))   # fg_j sits in w[t][jj] for jj < j <= t
        df[j] = float(dlog_f * sig(-fp[j]))
    return dict(H=H, dq=dq, dk=dk, dv=dv, di=di, df=df)


@pytest.mark.parametrize("variant", [EXP, SIG])
def test_p8_extreme_gate_preactivations_against_arbitrary_precision(variant):
    """Gate pre-activations far outside the benchmark's range (|x| up to 300: exp(i~) up to 1e130, forget gates
    down to 1e-130 and up to 1 - 1e-130, resets next to saturated steps): the stabilised fp64 recurrence, the
    quadratic form, the chunkwise form and the backward definitions against the unstabilised cell evaluated
    with 150 digits."""
    g = np.random.default_rng(80)
    S, T, dqk, dhv = 2, 9, 3, 2
    d = dict(q=g.standard_normal((S, T, dqk)), k=g.standard_normal((S, T, dqk)), v=g.standard_normal((S, T, dhv)),
             i_pre=np.array([[300.0, -300.0, 45.0, 0.0, -60.0, 120.0, 119.0, -5.0, 250.0],
                             [-250.0, -249.0, -300.0, 10.0, 80.0, -80.0, 0.5, 299.0, -299.0]]),
             f_pre=np.array([[0.0, 300.0, -300.0, 50.0, -50.0, 3.0, 200.0, -120.0, 1.0],
                             [300.0, 299.0, 60.0, -300.0, -2.0, 40.0, -40.0, 100.0, -100.0]]),
             C0=None, n0=None, m0=None)
    dH = g.standard_normal((S, T, dhv))
    rec = orc.recurrent_fwd(**d, variant=variant, eps=0.0)
    quad = orc.quadratic_fwd(**d, variant=variant, eps=0.0)
    bq = orc.quadratic_bwd(**d, dH=dH, variant=variant, eps=0.0)
    for L in (1, 3, 9):
        ch = orc.chunkwise_fwd(**d, variant=variant, eps=0.0, chunk=L)
        bc = orc.chunkwise_bwd(**d, dH=dH, variant=variant, eps=0.0, chunk=L)
        for s in range(S):
            ref = _mp_cell(d, dH, variant, s)
            for got in (rec["H"][s], quad["H"][s], ch["H"][s]):
                assert np.all(np.isfinite(got))
                close(got, ref["H"], 1e-11)
            for b in (bq, bc):
                for name in ("dq", "dk", "dv", "di", "df"):
                    assert np.all(np.isfinite(b[name][s])), name
                    close(b[name][s], ref[name], 1e-10)
