"""TEST INFRASTRUCTURE ONLY -- fp64 CPU oracle for what surrounds the mLSTM cell in a layer.

Plain numpy evaluations, written from the paper's equations; nothing is shared
with (or imported from) the HIP path.  Only tests, the smoke check and the
benchmark's cpu_baseline leg may import this module.

  softcap            c * tanh(x / c) on the gate pre-activations (soft-capping
                     equation of App. E, "Training details"; c = 15 there).
  norm_fwd           the NORM of the hidden-state output equation (last line of
                     the mLSTM equations in Sec. 2.1), per head over d_hv:
                     RMS norm as written out in Sec. 4.1
                     (y = x / sqrt(mean(x^2) + eps) (.) gamma), or LayerNorm
                     (subtract the mean, divide by sqrt(var + eps), scale, shift).
  norm_gate_fwd      h = sigma(o~) (.) NORM(h~)   (Sec. 2.1, output gate o = sigma(o~)).
  norm_gate_bwd      exact derivative of norm_gate_fwd (no approximation is
                     involved in this part of the layer).
  layer_fwd/_bwd     soft-cap -> mLSTM cell (mlstm_oracle) -> NORM -> output gate,
                     and the chain rule through it; the cell's own backward is the
                     paper's (normaliser held constant, App. B.3).
  transfer_gain      G_before, G_after of the gain equation in Sec. 4.1 ("Transfer
                     Behavior of the mLSTM"): max-norm of h~_t (resp. NORM(h~_t))
                     over max-norm of v_t, averaged over time.

Layout: hidden states (B, NH, T, dhv); gamma, beta (NH, dhv) -- every head has
its own scale ("multi-head" norm); o~ like the hidden states.
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np

from . import mlstm_oracle as cell

RMS, LAYER = 0, 1


def softcap(x, c):
    """c * tanh(x / c); c <= 0 or None switches it off."""
    x = np.asarray(x, dtype=np.float64)
    if c is None or c <= 0:
        return x.copy()
    return c * np.tanh(x / c)


def softcap_grad(x, c):
    x = np.asarray(x, dtype=np.float64)
    if c is None or c <= 0:
        return np.ones_like(x)
    t = np.tanh(x / c)
    return 1.0 - t * t


def _stats(x, kind, eps):
    d = x.shape[-1]
    if kind == RMS:
        mu = np.zeros(x.shape[:-1] + (1,))
        r = 1.0 / np.sqrt((x * x).sum(-1, keepdims=True) / d + eps)
    elif kind == LAYER:
        mu = x.sum(-1, keepdims=True) / d
        xc = x - mu
        r = 1.0 / np.sqrt((xc * xc).sum(-1, keepdims=True) / d + eps)
    else:
        raise ValueError("unknown norm kind")
    return mu, r


def norm_fwd(x, gamma=None, beta=None, kind=RMS, eps=1e-6):
    """x: (B, NH, T, d); gamma, beta: (NH, d) or None (1 and 0)."""
    x = np.asarray(x, dtype=np.float64)
    mu, r = _stats(x, kind, eps)
    y = (x - mu) * r
    if gamma is not None:
        y = y * np.asarray(gamma, dtype=np.float64)[None, :, None, :]
    if beta is not None and kind == LAYER:
        y = y + np.asarray(beta, dtype=np.float64)[None, :, None, :]
    return y


def norm_gate_fwd(h, o_pre=None, gamma=None, beta=None, kind=RMS, eps=1e-6):
    y = norm_fwd(h, gamma, beta, kind, eps)
    if o_pre is not None:
        y = cell.sigmoid(o_pre) * y
    return y


def norm_gate_bwd(h, dy, o_pre=None, gamma=None, beta=None, kind=RMS, eps=1e-6) -> Dict[str, Optional[np.ndarray]]:
    """Returns dh (like h), do_pre (like h, or None), dgamma, dbeta ((NH, d); dbeta None for RMS)."""
    h = np.asarray(h, dtype=np.float64)
    dy = np.asarray(dy, dtype=np.float64)
    d = h.shape[-1]
    mu, r = _stats(h, kind, eps)
    xh = (h - mu) * r                                   # normalised, before scale and shift
    g = 1.0 if gamma is None else np.asarray(gamma, dtype=np.float64)[None, :, None, :]
    nrm = xh * g
    if beta is not None and kind == LAYER:
        nrm = nrm + np.asarray(beta, dtype=np.float64)[None, :, None, :]
    if o_pre is not None:
        o = cell.sigmoid(o_pre)
        do_pre = dy * nrm * o * (1.0 - o)
        dn = dy * o
    else:
        do_pre = None
        dn = dy
    dgamma = (dn * xh).sum(axis=(0, 2))
    dbeta = dn.sum(axis=(0, 2)) if kind == LAYER else None
    dxh = dn * g
    if kind == RMS:
        dh = r * (dxh - xh * (dxh * xh).sum(-1, keepdims=True) / d)
    else:
        dh = r * (dxh - dxh.sum(-1, keepdims=True) / d - xh * (dxh * xh).sum(-1, keepdims=True) / d)
    return dict(dh=dh, do_pre=do_pre, dgamma=dgamma, dbeta=dbeta)


def _slices(a):
    a = np.asarray(a, dtype=np.float64)
    return a.reshape((-1,) + a.shape[2:])


def layer_fwd(q, k, v, i_pre, f_pre, o_pre=None, gamma=None, beta=None, variant=cell.EXP, eps=1e-6,
              gate_softcap=0.0, kind=RMS, norm_eps=1e-6) -> Dict[str, np.ndarray]:
    """(B, NH, T, .) inputs.  Returns y (the layer output), H (the cell output h~) and n_out, m_out."""
    B, NH = np.asarray(q).shape[:2]
    ic, fc = softcap(i_pre, gate_softcap), softcap(f_pre, gate_softcap)
    o = cell.recurrent_fwd(_slices(q), _slices(k), _slices(v), _slices(ic), _slices(fc), variant=variant, eps=eps)
    H = o["H"].reshape((B, NH) + o["H"].shape[1:])
    y = norm_gate_fwd(H, o_pre, gamma, beta, kind, norm_eps)
    return dict(y=y, H=H, n_out=o["n_out"].reshape(B, NH, -1), m_out=o["m_out"].reshape(B, NH, -1))


def layer_bwd(q, k, v, i_pre, f_pre, dy, o_pre=None, gamma=None, beta=None, variant=cell.EXP, eps=1e-6,
              gate_softcap=0.0, kind=RMS, norm_eps=1e-6, chunk=64) -> Dict[str, Optional[np.ndarray]]:
    B, NH = np.asarray(q).shape[:2]
    f = layer_fwd(q, k, v, i_pre, f_pre, o_pre, gamma, beta, variant, eps, gate_softcap, kind, norm_eps)
    ng = norm_gate_bwd(f["H"], dy, o_pre, gamma, beta, kind, norm_eps)
    ic, fc = softcap(i_pre, gate_softcap), softcap(f_pre, gate_softcap)
    g = cell.chunkwise_bwd(_slices(q), _slices(k), _slices(v), _slices(ic), _slices(fc), _slices(ng["dh"]),
                           variant=variant, eps=eps, chunk=chunk)
    shp = lambda a: a.reshape((B, NH) + a.shape[1:])
    out = dict(dq=shp(g["dq"]), dk=shp(g["dk"]), dv=shp(g["dv"]),
               d_i_pre=shp(g["di"]) * softcap_grad(i_pre, gate_softcap),
               d_f_pre=shp(g["df"]) * softcap_grad(f_pre, gate_softcap),
               do_pre=ng["do_pre"], dgamma=ng["dgamma"], dbeta=ng["dbeta"], dh=ng["dh"])
    return out


def transfer_gain(h, v, kind=RMS, norm_eps=1e-6):
    """h, v: (B, NH, T, d).  Returns (G_before, G_after), each (B, NH): time averages of the ratios of
    max-norms; the norm layer has unit scale and no shift."""
    h = np.asarray(h, dtype=np.float64); v = np.asarray(v, dtype=np.float64)
    vmax = np.abs(v).max(-1)
    gb = (np.abs(h).max(-1) / vmax).mean(-1)
    ga = (np.abs(norm_fwd(h, None, None, kind, norm_eps)).max(-1) / vmax).mean(-1)
    return gb, ga
