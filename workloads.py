"""Seeded synthetic inputs for the mLSTM / mLSTMsig kernel path.

This module only *draws numbers*: it holds none of the method's arithmetic
(no gates, no recurrences).  Both the fp64 CPU oracle and the HIP path read
their inputs from here so that they see identical bits.

The paper's kernel benchmarks use synthetic tensors of the shapes of its
language models (Sec. 5.1, App. E.3: 8 heads, d_qk=256, d_hv=512 for the
7B-shaped head).  The distributions below are the ones the benchmark
configurations name: q, k, v ~ N(0,1); input-gate pre-activation ~ N(0,1);
forget-gate pre-activation ~ N(3,1) (N(5,1) for the long-memory case);
initial states C0, n0 ~ N(0, std 0.1), m0 = 0; upstream gradients ~ N(0,1).
"""
from __future__ import annotations

import dataclasses
from typing import Dict, Optional

import numpy as np

EXP, SIG = 0, 1          # variant codes (exponential / sigmoid input gate)
F32, BF16 = 0, 1         # dtype codes of q, k, v, H and their gradients


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    B: int
    NH: int
    T: int
    dqk: int
    dhv: int
    chunk: int
    variant: int
    dtype: int
    f_mean: float = 3.0
    init_state: bool = False
    backward: bool = False
    seed: int = 1000

    @property
    def tokens(self) -> int:
        return self.B * self.T


# The five benchmark configurations (index = position in the configs list).
CONFIGS: Dict[str, Workload] = {
    "c0": Workload("c0", 1, 1, 256, 64, 64, 64, EXP, F32, seed=1000),
    "c1": Workload("c1", 4, 8, 2048, 128, 128, 128, EXP, BF16, init_state=True, seed=1001),
    "c2": Workload("c2", 1, 8, 8192, 256, 512, 256, SIG, BF16, seed=1002),
    "c3": Workload("c3", 1, 8, 32768, 256, 512, 512, EXP, BF16, f_mean=5.0, seed=1003),
    "c4": Workload("c4", 2, 8, 8192, 256, 512, 256, EXP, BF16, backward=True, seed=1004),
    "c4sig": Workload("c4sig", 2, 8, 8192, 256, 512, 256, SIG, BF16, backward=True, seed=1004),
}
C2_CHUNKS = (64, 128, 256, 512, 1024)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bfloat16 (ties to even); returns fp32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    r = ((u + bias) & np.uint32(0xFFFF0000)).astype(np.uint32)
    return r.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of values that are already bf16-representable."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return (u >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


def make_inputs(w: Workload, heads: Optional[int] = None, slices=None) -> Dict[str, np.ndarray]:
    """Draw the input tensors of a workload (fp32 arrays; bf16 workloads are
    already rounded to bf16-representable values, so the oracle and the kernel
    both start from the same quantised inputs).

    heads: if given, only the first `heads` (batch*head) slices are drawn
    and returned with shape (1, heads, ...); slice s of the full problem is
    drawn from its own stream (seed, s), so the subset equals the full draw.
    slices: instead of `heads`, an explicit list of (batch*head) slice indices
    (b * NH + h), returned in that order with shape (1, len(slices), ...).
    """
    BH = w.B * w.NH
    if slices is not None:
        idx = [int(s) for s in slices]
        assert heads is None and all(0 <= s < BH for s in idx)
    else:
        idx = list(range(BH if heads is None else min(heads, BH)))
    n = len(idx)
    shp = (w.B, w.NH) if (heads is None and slices is None) else (1, n)

    def draw(tag: int, tail, mean=0.0, std=1.0):
        out = np.empty((n,) + tuple(tail), dtype=np.float32)
        for j, s in enumerate(idx):
            g = np.random.Generator(np.random.Philox(key=w.seed, counter=[tag, s, 0, 0]))
            out[j] = g.standard_normal(tail, dtype=np.float32) * np.float32(std) + np.float32(mean)
        return out.reshape(shp + tuple(tail))

    q = draw(1, (w.T, w.dqk))
    k = draw(2, (w.T, w.dqk))
    v = draw(3, (w.T, w.dhv))
    if w.dtype == BF16:
        q, k, v = bf16_round(q), bf16_round(k), bf16_round(v)
    d = {
        "q": q, "k": k, "v": v,
        "i_pre": draw(4, (w.T,)),
        "f_pre": draw(5, (w.T,), mean=w.f_mean),
    }
    if w.init_state:
        d["C0"] = draw(6, (w.dqk, w.dhv), std=0.1)
        d["n0"] = draw(7, (w.dqk,), std=0.1)
        d["m0"] = np.zeros(shp, dtype=np.float32)
    if w.backward:
        dH = draw(8, (w.T, w.dhv))
        d["dH"] = bf16_round(dH) if w.dtype == BF16 else dH
    return d


def make_layer_inputs(w: Workload, heads: Optional[int] = None, gate_scale: float = 1.0) -> Dict[str, np.ndarray]:
    """The inputs of make_inputs plus what the layer around the cell reads: output-gate
    pre-activations o_pre ~ N(0,1) shaped like v, norm scale gamma ~ 1 + N(0, std 0.1) and shift
    beta ~ N(0, std 0.1) per head, an upstream gradient dY ~ N(0,1) (stored under "dH" by
    make_inputs).  gate_scale multiplies both gate pre-activations (to reach the range where a
    soft-cap matters).  With `heads`, the first `heads` slices must belong to one batch element."""
    d = make_inputs(w, heads)
    BH = w.B * w.NH
    n = BH if heads is None else min(heads, BH)
    assert heads is None or n <= w.NH
    shp = (w.B, w.NH) if heads is None else (1, n)
    o = np.empty((n, w.T, w.dhv), dtype=np.float32)
    for s in range(n):
        g = np.random.Generator(np.random.Philox(key=w.seed, counter=[9, s, 0, 0]))
        o[s] = g.standard_normal((w.T, w.dhv), dtype=np.float32)
    o = o.reshape(shp + (w.T, w.dhv))
    d["o_pre"] = bf16_round(o) if w.dtype == BF16 else o
    nh = w.NH if heads is None else n
    gam = np.empty((nh, w.dhv), dtype=np.float32); bet = np.empty((nh, w.dhv), dtype=np.float32)
    for h in range(nh):
        g = np.random.Generator(np.random.Philox(key=w.seed, counter=[10, h, 0, 0]))
        gam[h] = np.float32(1.0) + np.float32(0.1) * g.standard_normal((w.dhv,), dtype=np.float32)
        bet[h] = np.float32(0.1) * g.standard_normal((w.dhv,), dtype=np.float32)
    d["gamma"] = gam; d["beta"] = bet
    if gate_scale != 1.0:
        d["i_pre"] = (d["i_pre"] * np.float32(gate_scale)).astype(np.float32)
        d["f_pre"] = (d["f_pre"] * np.float32(gate_scale)).astype(np.float32)
    return d


def small(variant: int, dtype: int, B=1, NH=2, T=256, dqk=64, dhv=128, chunk=64,
          seed=7, init_state=True, backward=True, f_mean=3.0) -> Workload:
    """A reduced workload of the same recipe for parity tests."""
    return Workload("small", B, NH, T, dqk, dhv, chunk, variant, dtype,
                    f_mean=f_mean, init_state=init_state, backward=backward, seed=seed)


# ---- moving a drawn workload to the device / to the oracle's layout (no arithmetic) ----------------
def to_dev(a, dtype):
    """numpy array -> device tensor; bf16 workloads are bf16-representable already, so the cast is exact."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t.to(torch.bfloat16) if dtype == BF16 else t


def dev_inputs(w: Workload, d: Dict[str, np.ndarray]):
    return {key: to_dev(val, w.dtype if key in ("q", "k", "v", "dH", "o_pre") else F32) for key, val in d.items()}


def flat(a) -> np.ndarray:
    """(B, NH, ...) -> (B*NH, ...) float64, the layout the oracle takes."""
    a = np.asarray(a, dtype=np.float64)
    return a.reshape((a.shape[0] * a.shape[1],) + a.shape[2:])


def oracle_inputs(d: Dict[str, np.ndarray]):
    keys = ("q", "k", "v", "i_pre", "f_pre", "C0", "n0", "m0")
    return {k_: (flat(d[k_]) if k_ in d else None) for k_ in keys}
