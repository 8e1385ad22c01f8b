"""TEST INFRASTRUCTURE ONLY -- fp64 CPU oracle for the mLSTM / mLSTMsig path.

Plain, slow, double-precision evaluations of what the kernels compute, written
from the paper's equations.  Nothing here is tuned, tiled or fused, and nothing
is shared with (or imported from) the HIP path.  Only tests, the smoke check
and the benchmark's cpu_baseline leg may import this module.

Contents (all arrays float64, one (batch*head) slice = leading axis):
  recurrent_fwd      step-by-step recurrence, paper Sec. 2.1 (mLSTMexp) and
                     Sec. 4.1 (mLSTMsig); implemented in C (mlstm_recurrent.c).
                     This is the definition of the forward result.
  quadratic_fwd      fully parallel formulation, paper App. B.1, extended by an
                     initial state (the extension follows from unrolling the
                     recurrence of Sec. 2.1).
  chunkwise_fwd      chunkwise-parallel formulation, paper App. B.2, any chunk
                     size L (ragged last chunk allowed).
  quadratic_bwd      definition of the backward result: the gradient of
                     sum<dH,H> + <dCn,C_T> with the normaliser (h_denom) and all
                     max states held constant (paper App. B.3, first paragraph).
  chunkwise_bwd      chunkwise-parallel backward pass, paper App. B.3.

Readings of the paper (each also listed in the design notes):
  * chunk k covers steps (k-1)L+1..kL (the text's index range with N_c is a typo);
  * the factor exp(m_intra - m_combine) scales the *intra* parts and
    Q-bar = b-bar (.) Q/sqrt(d) (App. C.2's last two equations), not the way
    Alg. 1's last lines print it;
  * n_k = g-bar n_{k-1} + K-bar^T 1 (the simplified form's "K-bar^T V" is a typo);
  * in App. B.3 the three lines "delta f-bar = ..." are contributions that add:
    delta f-bar_s = delta g + sum_{j>=s} delta b_j + sum_{j<s} delta a_j
    (the a-term is an exclusive forward cumulative sum because a_j collects
    f-bar_s for s>j), and the gradient w.r.t. the *log* gate matrix is
    delta S-bar (.) S-bar (the printed delta D = delta S-bar (.) S is the gradient
    w.r.t. D itself);
  * mLSTMsig in parallel/chunkwise form: i-bar = log sigma(i~), no max state,
    normaliser 1 (App. D.2, "Normalizers of mLSTMexp and mLSTMsig");
  * eps is added to max{|n^T q~|, exp(-m)}; eps = 0 is the paper's formula.

Gate pre-activations far outside the benchmark's ranges (|x| up to 300) are pinned
against the unstabilised cell evaluated in 150-digit arithmetic (pin P8 of the tests).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, Optional

import numpy as np

EXP, SIG = 0, 1
_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mlstm_recurrent.c")
_LIB = os.path.join(_HERE, "liboracle_mlstm.so")
_lib = None


def build_c(force: bool = False) -> str:
    """Compile the C part of the oracle with gcc (OpenMP over batch*head)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build_c()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        lib.oracle_mlstm_recurrent_fwd.restype = ctypes.c_int
        lib.oracle_mlstm_recurrent_fwd.argtypes = [dp] * 8 + [ctypes.c_long] * 4 + [ctypes.c_int, ctypes.c_double] + [dp] * 6
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _f64(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def log_sigmoid(x):
    x = np.asarray(x, dtype=np.float64)
    return np.minimum(x, 0.0) - np.log1p(np.exp(-np.abs(x)))


def sigmoid(x):
    return np.exp(log_sigmoid(x))


# --------------------------------------------------------------------------
# forward: recurrence (definition), Sec. 2.1 / Sec. 4.1
# --------------------------------------------------------------------------
def recurrent_fwd(q, k, v, i_pre, f_pre, C0=None, n0=None, m0=None, variant=EXP, eps=0.0) -> Dict[str, np.ndarray]:
    """q,k: (S,T,dqk); v: (S,T,dhv); gates (S,T); states (S,dqk,dhv),(S,dqk),(S)."""
    q, k, v, i_pre, f_pre = map(_f64, (q, k, v, i_pre, f_pre))
    C0, n0, m0 = _f64(C0), _f64(n0), _f64(m0)
    S, T, dqk = q.shape
    dhv = v.shape[-1]
    H = np.empty((S, T, dhv)); Cn = np.empty((S, dqk, dhv)); nn = np.empty((S, dqk)); mn = np.empty((S,))
    n_out = np.empty((S, T)); m_out = np.empty((S, T))
    rc = _load().oracle_mlstm_recurrent_fwd(_p(q), _p(k), _p(v), _p(i_pre), _p(f_pre), _p(C0), _p(n0), _p(m0),
                                            S, T, dqk, dhv, int(variant), float(eps),
                                            _p(H), _p(Cn), _p(nn), _p(mn), _p(n_out), _p(m_out))
    if rc != 0:
        raise MemoryError("oracle_mlstm_recurrent_fwd failed")
    return dict(H=H, Cn=Cn, nn=nn, mn=mn, n_out=n_out, m_out=m_out)


# --------------------------------------------------------------------------
# forward: fully parallel (quadratic) formulation, App. B.1
# --------------------------------------------------------------------------
def _quadratic_weights(i_pre, f_pre, m0, variant):
    """Log-weights of one slice.  Returns (Dt, z, m): Dt[t,j] = sum_{s=j+1..t} f-bar_s
    + i-bar_j for j<=t (-inf above the diagonal), z[t] = sum_{s<=t} f-bar_s + m0 (the
    log-weight of the initial state), m[t] the row max (0 for the sigmoid variant)."""
    T = i_pre.shape[0]
    fbar = log_sigmoid(f_pre)
    ibar = i_pre if variant == EXP else log_sigmoid(i_pre)
    cumF = np.cumsum(fbar)
    Dt = cumF[:, None] - cumF[None, :] + ibar[None, :]
    Dt = np.where(np.tril(np.ones((T, T), dtype=bool)), Dt, -np.inf)
    z = cumF + (m0 if variant == EXP else 0.0)
    if variant == EXP:
        m = np.maximum(Dt.max(axis=1), z)
    else:
        m = np.zeros(T)
    return Dt, z, m, cumF, ibar


def quadratic_fwd(q, k, v, i_pre, f_pre, C0=None, n0=None, m0=None, variant=EXP, eps=0.0):
    q, k, v, i_pre, f_pre = map(_f64, (q, k, v, i_pre, f_pre))
    S, T, dqk = q.shape
    dhv = v.shape[-1]
    H = np.empty((S, T, dhv)); n_out = np.zeros((S, T)); m_out = np.zeros((S, T))
    for s in range(S):
        m0s = 0.0 if m0 is None else float(m0[s])
        Dt, z, m, _, _ = _quadratic_weights(i_pre[s], f_pre[s], m0s, variant)
        D = np.exp(Dt - m[:, None])                       # D = exp(D~ - m)
        Sm = (q[s] @ k[s].T) / np.sqrt(dqk)               # S = Q K^T / sqrt(d_qk)
        Sbar = Sm * D                                     # S-bar = S (.) D
        num = Sbar @ v[s]
        nrm = Sbar.sum(axis=1)
        if C0 is not None:
            w0 = np.exp(z - m)
            qs = q[s] / np.sqrt(dqk)
            num = num + w0[:, None] * (qs @ _f64(C0[s]))
            if n0 is not None:
                nrm = nrm + w0 * (qs @ _f64(n0[s]))
        if variant == EXP:
            den = np.maximum(np.abs(nrm), np.exp(-m)) + eps   # n = max(|S-bar 1|, exp(-m))
            n_out[s] = nrm; m_out[s] = m
        else:
            den = np.ones(T)
        H[s] = num / den[:, None]
    return dict(H=H, n_out=n_out, m_out=m_out)


# --------------------------------------------------------------------------
# forward: chunkwise-parallel formulation, App. B.2
# --------------------------------------------------------------------------
def chunk_gates(i_pre, f_pre, variant):
    """Chunkwise log gates of one chunk (App. B.2, 'Chunkwise Gates'):
    g = sum f-bar, b = cumsum f-bar, a_j = sum_{s>j} f-bar_s + i-bar_j (formed as a
    shifted reverse cumulative sum, not as g - b)."""
    fbar = log_sigmoid(f_pre)
    ibar = i_pre if variant == EXP else log_sigmoid(i_pre)
    b = np.cumsum(fbar)
    g = b[-1]
    rev = np.concatenate([np.cumsum(fbar[1:][::-1])[::-1], [0.0]])
    a = rev + ibar
    return g, b, a, ibar


def chunkwise_fwd(q, k, v, i_pre, f_pre, C0=None, n0=None, m0=None, variant=EXP, eps=0.0, chunk=64,
                  return_states=False):
    q, k, v, i_pre, f_pre = map(_f64, (q, k, v, i_pre, f_pre))
    S, T, dqk = q.shape
    dhv = v.shape[-1]
    L = int(chunk)
    H = np.empty((S, T, dhv)); n_out = np.zeros((S, T)); m_out = np.zeros((S, T))
    Cn = np.empty((S, dqk, dhv)); nn = np.zeros((S, dqk)); mn = np.zeros((S,))
    states = []
    for s in range(S):
        C = np.zeros((dqk, dhv)) if C0 is None else _f64(C0[s]).copy()
        n = np.zeros(dqk) if n0 is None else _f64(n0[s]).copy()
        m = 0.0 if (m0 is None or variant == SIG) else float(m0[s])
        st = []
        for t0 in range(0, T, L):
            t1 = min(t0 + L, T)
            Q = q[s, t0:t1] / np.sqrt(dqk); K = k[s, t0:t1]; V = v[s, t0:t1]
            g, b, a, ibar = chunk_gates(i_pre[s, t0:t1], f_pre[s, t0:t1], variant)
            st.append((C.copy(), n.copy(), m))
            Lc = t1 - t0
            # intra-chunk: D~_ij = b_i - b_j + i-bar_j (i >= j)
            Dt = b[:, None] - b[None, :] + ibar[None, :]
            Dt = np.where(np.tril(np.ones((Lc, Lc), dtype=bool)), Dt, -np.inf)
            if variant == EXP:
                m_intra = Dt.max(axis=1)
                m_comb = np.maximum(b + m, m_intra)            # m_combine
            else:
                m_comb = np.zeros(Lc)
            bbar = np.exp(b + m - m_comb)                      # b-bar
            Sbar = (Q @ K.T) * np.exp(Dt - m_comb[:, None])
            num = (bbar[:, None] * Q) @ C + Sbar @ V           # H_inter + H_intra
            if variant == EXP:
                nrm = (bbar[:, None] * Q) @ n + Sbar.sum(axis=1)
                den = np.maximum(np.abs(nrm), np.exp(-m_comb)) + eps
                n_out[s, t0:t1] = nrm; m_out[s, t0:t1] = m_comb
            else:
                den = np.ones(Lc)
            H[s, t0:t1] = num / den[:, None]
            # inter-chunk recurrence: m_k, C_k, n_k
            m_next = max(g + m, a.max()) if variant == EXP else 0.0
            gbar = np.exp(g + m - m_next)
            abar = np.exp(a - m_next)
            C = gbar * C + (abar[:, None] * K).T @ V
            n = gbar * n + (abar[:, None] * K).sum(axis=0)
            m = m_next
        Cn[s] = C
        if variant == EXP:
            nn[s] = n; mn[s] = m
        states.append(st)
    out = dict(H=H, Cn=Cn, nn=nn, mn=mn, n_out=n_out, m_out=m_out)
    if return_states:
        out["states"] = states
    return out


# --------------------------------------------------------------------------
# backward: definition (quadratic form), normaliser and max states held constant
# --------------------------------------------------------------------------
def quadratic_bwd(q, k, v, i_pre, f_pre, dH, C0=None, n0=None, m0=None, dCn=None, variant=EXP, eps=0.0):
    """Gradient of  l = sum_t <dH_t, H_t> + <dCn, C_T>  w.r.t. q, k, v, i_pre, f_pre, C0,
    where H_t = Num_t / den_t with den_t (and every max state) treated as constants.
    C_T, C0, dCn, dC0 are in the stabilised coordinates of m_T resp. m0."""
    q, k, v, i_pre, f_pre, dH = map(_f64, (q, k, v, i_pre, f_pre, dH))
    S, T, dqk = q.shape
    dhv = v.shape[-1]
    fwd = quadratic_fwd(q, k, v, i_pre, f_pre, C0, n0, m0, variant, eps)
    dq = np.zeros_like(q); dk = np.zeros_like(k); dv = np.zeros_like(v)
    di = np.zeros_like(i_pre); df = np.zeros_like(f_pre); dC0 = np.zeros((S, dqk, dhv))
    rs = 1.0 / np.sqrt(dqk)
    for s in range(S):
        m0s = 0.0 if (m0 is None or variant == SIG) else float(m0[s])
        Dt, z, m, cumF, ibar = _quadratic_weights(i_pre[s], f_pre[s], m0s, variant)
        if variant == EXP:
            den = np.maximum(np.abs(fwd["n_out"][s]), np.exp(-m)) + eps
        else:
            den = np.ones(T)
        W = np.exp(Dt - m[:, None])                  # weights of (t, j)
        w0 = np.exp(z - m)                           # weight of the initial state at step t
        dN = dH[s] / den[:, None]                    # gradient w.r.t. the numerator
        qs = q[s] * rs
        Sm = qs @ k[s].T                             # s_tj
        P = dN @ v[s].T                              # P_tj = <dN_t, v_j>
        dv[s] = (W * Sm).T @ dN
        dq[s] = ((W * P) @ k[s]) * rs
        dk[s] = (W * P).T @ qs
        E = W * Sm * P                               # gradient w.r.t. the log-weight D~_tj
        e0 = np.zeros(T)
        if C0 is not None:
            C0s = _f64(C0[s])
            dq[s] += (w0[:, None] * (dN @ C0s.T)) * rs
            e0 = w0 * np.einsum("td,td->t", qs @ C0s, dN)
            dC0[s] = (w0[:, None] * qs).T @ dN
        G = np.zeros(T); G0 = 0.0
        if dCn is not None:
            # C_T = sum_j exp(sum_{s>j} f-bar_s + i-bar_j - m_T) k_j v_j^T + exp(sum f-bar + m0 - m_T) C0
            mT = m[-1]
            wT = np.exp(cumF[-1] - cumF + ibar - mT)
            wT0 = np.exp(cumF[-1] + m0s - mT)
            dCs = _f64(dCn[s])
            dv[s] += wT[:, None] * (k[s] @ dCs)
            dk[s] += wT[:, None] * (v[s] @ dCs.T)
            G = wT * np.einsum("td,de,te->t", k[s], dCs, v[s])
            dC0[s] += wT0 * dCs
            if C0 is not None:
                G0 = wT0 * np.sum(_f64(C0[s]) * dCs)
        # i-bar_j enters the log-weight of every (t, j), t >= j, and of the final state
        dibar = E.sum(axis=0) + G
        # f-bar_s enters the log-weight of (t, j) for j < s <= t, of the initial-state
        # term for s <= t, and of the final state's term j for j < s (and of its C0 term)
        colcum = np.cumsum(E, axis=1)                # colcum[t, s] = sum_{j<=s} E[t, j]
        dfbar = np.zeros(T)
        for sidx in range(T):
            inner = colcum[sidx:, sidx - 1].sum() if sidx > 0 else 0.0
            dfbar[sidx] = inner + e0[sidx:].sum() + G[:sidx].sum() + G0
        di[s] = dibar if variant == EXP else dibar * sigmoid(-i_pre[s])
        df[s] = dfbar * sigmoid(-f_pre[s])
    return dict(dq=dq, dk=dk, dv=dv, di=di, df=df, dC0=dC0)


# --------------------------------------------------------------------------
# backward: chunkwise-parallel formulation, App. B.3
# --------------------------------------------------------------------------
def chunkwise_bwd(q, k, v, i_pre, f_pre, dH, C0=None, n0=None, m0=None, dCn=None, variant=EXP, eps=0.0,
                  chunk=64):
    q, k, v, i_pre, f_pre, dH = map(_f64, (q, k, v, i_pre, f_pre, dH))
    S, T, dqk = q.shape
    dhv = v.shape[-1]
    L = int(chunk)
    fwd = chunkwise_fwd(q, k, v, i_pre, f_pre, C0, n0, m0, variant, eps, L, return_states=True)
    dq = np.zeros_like(q); dk = np.zeros_like(k); dv = np.zeros_like(v)
    di = np.zeros_like(i_pre); df = np.zeros_like(f_pre); dC0 = np.zeros((S, dqk, dhv))
    rs = 1.0 / np.sqrt(dqk)
    for s in range(S):
        st = fwd["states"][s]
        starts = list(range(0, T, L))
        m_after = [st[i + 1][2] for i in range(len(starts) - 1)] + [float(fwd["mn"][s])]
        dC = np.zeros((dqk, dhv)) if dCn is None else _f64(dCn[s]).copy()   # delta C_k
        for ci in range(len(starts) - 1, -1, -1):
            t0 = starts[ci]; t1 = min(t0 + L, T); Lc = t1 - t0
            Cprev, _, mprev = st[ci]
            mk = m_after[ci] if variant == EXP else 0.0
            Q = q[s, t0:t1]; K = k[s, t0:t1]; V = v[s, t0:t1]
            g, b, a, ibar = chunk_gates(i_pre[s, t0:t1], f_pre[s, t0:t1], variant)
            if variant == EXP:
                m_comb = fwd["m_out"][s, t0:t1]
                den = np.maximum(np.abs(fwd["n_out"][s, t0:t1]), np.exp(-m_comb)) + eps
            else:
                m_comb = np.zeros(Lc); den = np.ones(Lc)
            gbar = np.exp(g + mprev - mk); abar = np.exp(a - mk); bbar = np.exp(b + mprev - m_comb)
            dHt = dH[s, t0:t1] / den[:, None]                       # delta H~ = delta H / h_denom
            # inter-chunk part
            Kbar = abar[:, None] * K
            dV_inter = Kbar @ dC                                     # K-bar dC_k
            dKbar = V @ dC.T                                         # V dC_k^T
            dK_inter = dKbar * abar[:, None]
            dQbar = dHt @ Cprev.T                                    # dH~ C_{k-1}^T
            dQ_inter = dQbar * bbar[:, None] * rs
            dg = np.sum(Cprev * dC) * gbar                           # delta g
            da = np.einsum("ld,ld->l", dKbar, K) * abar              # delta a
            db = np.einsum("ld,ld->l", dQbar, Q * rs) * bbar         # delta b (inter)
            dC_prev = gbar * dC + (bbar[:, None] * Q * rs).T @ dHt   # delta C_{k-1}
            # intra-chunk part
            Dt = b[:, None] - b[None, :] + ibar[None, :]
            Dt = np.where(np.tril(np.ones((Lc, Lc), dtype=bool)), Dt, -np.inf)
            D = np.exp(Dt - m_comb[:, None])
            Sm = (Q @ K.T) * rs
            Sbar = Sm * D
            dV_intra = Sbar.T @ dHt
            dSbar = dHt @ V.T
            dS = dSbar * D
            dQ_intra = (dS @ K) * rs
            dK_intra = (dS.T @ Q) * rs
            dDt = dSbar * Sbar                                       # gradient w.r.t. the log gate matrix
            db_q = dDt.sum(axis=1)
            db_kv = -dDt.sum(axis=0)
            di_intra = dDt.sum(axis=0)
            # combine
            dq[s, t0:t1] = dQ_inter + dQ_intra
            dk[s, t0:t1] = dK_inter + dK_intra
            dv[s, t0:t1] = dV_inter + dV_intra
            db_all = db + db_q + db_kv
            dfbar = dg + np.cumsum(db_all[::-1])[::-1] + (np.cumsum(da) - da)
            dibar = da + di_intra
            di[s, t0:t1] = dibar if variant == EXP else dibar * sigmoid(-i_pre[s, t0:t1])
            df[s, t0:t1] = dfbar * sigmoid(-f_pre[s, t0:t1])
            dC = dC_prev
        dC0[s] = dC
    return dict(dq=dq, dk=dk, dv=dv, di=di, df=df, dC0=dC0)
