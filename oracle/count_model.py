"""TEST INFRASTRUCTURE ONLY -- the paper's FLOP / byte count model (App. F, App. G).

Closed forms for the chunkwise-parallel mLSTM forward pass, per head and for a
full sequence of length T, with every per-operation factor F_OP set to 1 as in
the paper's simplified tables.  Used to pin the measurement model (the numbers
the paper prints for it) and as the reference for the algorithmic FLOP counts
the benchmark reports.  Not used by the kernels.
"""
from __future__ import annotations

import math


def flops_chunkwise_sig(T, L, dqk, dhv, F_causal=0.5):
    """Total simplified FLOPs of mLSTMsig, chunkwise-parallel (App. F.2, table of
    total simplified FLOP counts, row 'chunkwise-parallel', column mLSTMsig)."""
    return (T * L * F_causal * (2 * (dqk + dhv) + 6) + T * L
            + T * (4 * dqk * dhv + 2 * dqk + dhv + 11)
            + (T / L) * (2 * dqk * dhv + 5))


def flops_chunkwise_exp(T, L, dqk, dhv, F_causal=0.5):
    """Same table, column mLSTMexp."""
    return (T * L * F_causal * (2 * (dqk + dhv) + 8) + T * L + 2 * T * F_causal
            + T * (4 * dqk * dhv + 6 * dqk + 4 * dhv + 13)
            + (T / L) * (2 * dqk * dhv + 2 * dqk + 5))


def flops_recurrent_sig(T, dqk, dhv):
    return T * (6 * dqk * dhv + dqk + 2)


def flops_recurrent_exp(T, dqk, dhv):
    return T * (6 * dqk * dhv + 7 * dqk + dhv + 12)


def flops_parallel_sig(T, dqk, dhv, F_causal=0.5):
    return T * T * F_causal * (2 * (dqk + dhv) + 2) + 6.5 * T * T + 4.5 * T


def flops_parallel_exp(T, dqk, dhv, F_causal=0.5):
    return T * T * F_causal * (2 * (dqk + dhv) + 6) + 2 * T * F_causal + 6.5 * T * T + 2.5 * T


def bytes_chunkwise_sig(T, L, dqk, dhv, bytes_qkv=2, bytes_if=2, bytes_Cmn=4):
    """Memory operations of mLSTMsig, chunkwise-parallel, two kernels (App. F.1, table
    of memory operation counts, 'Total' row), times the number of chunks."""
    per_chunk = 4 * L * bytes_if + 3 * L * (dhv + dqk) * bytes_qkv + 2 * dhv * dqk * bytes_Cmn
    return (T / L) * per_chunk


def bytes_chunkwise_exp(T, L, dqk, dhv, bytes_qkv=2, bytes_if=2, bytes_Cmn=4):
    per_chunk = (4 * L * bytes_if + 3 * L * (dhv + dqk) * bytes_qkv
                 + 2 * (L + dhv * dqk + dqk + 1) * bytes_Cmn)
    return (T / L) * per_chunk


def intensity_sig_closed_form(L, dhv, p_qk, F_causal=0.5, bytes_Cmn=4):
    """Arithmetic intensity of the mLSTMsig forward pass (App. G.2, the closed form)."""
    num = (L * L * F_causal * (2 * dhv * p_qk + 2 * dhv + 6) + L * L
           + L * (4 * dhv * dhv * p_qk + 2 * dhv * p_qk + dhv + 11) + 2 * dhv * dhv * p_qk + 5)
    den = 6 * L * dhv * (1 + p_qk) + 8 * L + 2 * bytes_Cmn * dhv * dhv * p_qk
    return num / den


def l_opt_flop(dhv, p_qk, F_causal=0.5):
    """FLOP-optimal chunk size (App. F.5)."""
    return math.sqrt((2 * dhv * dhv * p_qk + 5) / (2 * F_causal * (dhv * (1 + p_qk) + 3) + 1))


def l_opt_runtime(dhv, p_qk, I_acc, F_causal=0.5, bytes_Cmn=4):
    """Runtime-optimal chunk size (App. G.4)."""
    return math.sqrt((2 * dhv * dhv * p_qk + 5 + 2 * I_acc * dhv * dhv * p_qk * bytes_Cmn)
                     / (2 * F_causal * (dhv * (1 + p_qk) + 3) + 1))


def bytes_recurrent_step_exp(dqk, dhv, bytes_qkv=2, bytes_if=4, bytes_Cmn=4):
    """Memory operations of one step of the recurrent mLSTMexp for one head, states materialised
    after every step (App. F.2, memory operation counts of the recurrent formulation): loads
    q, k, v, the two gates and (C, n, m); stores h and (C, n, m)."""
    load = (2 * dqk + dhv) * bytes_qkv + 2 * bytes_if + (dqk * dhv + dqk + 1) * bytes_Cmn
    store = dhv * bytes_qkv + (dqk * dhv + dqk + 1) * bytes_Cmn
    return load + store


def bytes_recurrent_step_sig(dqk, dhv, bytes_qkv=2, bytes_if=4, bytes_Cmn=4):
    """The same for mLSTMsig: no normaliser and no max state."""
    load = (2 * dqk + dhv) * bytes_qkv + 2 * bytes_if + dqk * dhv * bytes_Cmn
    store = dhv * bytes_qkv + dqk * dhv * bytes_Cmn
    return load + store
