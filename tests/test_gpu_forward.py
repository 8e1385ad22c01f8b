"""GPU parity of tfla_mlstm_fwd against the fp64 oracle (recurrent formulation, Sec. 2.1 /
Sec. 4.1), element by element on seeded inputs.  Bar: max|gpu-ref|/max|ref| <= 2e-2 for bf16
inputs with fp32 accumulation, <= 1e-4 for the fp32 path."""
import numpy as np
import pytest

import workloads as wl
from oracle import mlstm_oracle as orc

pytestmark = pytest.mark.gpu


def run_case(w, heads=None):
    import paper_2503_14376_amd as tfla
    from tests import gpu_util as gu
    d = wl.make_inputs(w, heads)
    dev = gu.dev_inputs(w, d)
    out = tfla.mlstm_fwd(dev["q"], dev["k"], dev["v"], dev["i_pre"], dev["f_pre"],
                         dev.get("C0"), dev.get("n0"), dev.get("m0"), chunk=w.chunk, variant=w.variant, eps=1e-6)
    ref = orc.recurrent_fwd(**gu.oracle_inputs(d), variant=w.variant, eps=1e-6)
    errs = gu.check_fwd(w, d, out, ref)
    print(w.name, w.variant, w.dtype, w.T, w.dqk, w.dhv, w.chunk, errs, flush=True)
    return errs


@pytest.mark.parametrize("variant", [wl.EXP, wl.SIG])
@pytest.mark.parametrize("dtype", [wl.BF16, wl.F32])
@pytest.mark.parametrize("shape", [(256, 64, 64, 64), (512, 64, 128, 128), (512, 128, 64, 256), (384, 128, 128, 192)])
def test_fwd_small(variant, dtype, shape):
    T, dqk, dhv, chunk = shape
    run_case(wl.small(variant, dtype, B=1, NH=2, T=T, dqk=dqk, dhv=dhv, chunk=chunk, seed=11 + T + dqk))


@pytest.mark.parametrize("variant", [wl.EXP, wl.SIG])
def test_fwd_7b_head_shape_bf16(variant):
    run_case(wl.small(variant, wl.BF16, B=1, NH=1, T=1024, dqk=256, dhv=512, chunk=256, seed=21))


def test_fwd_config0():
    run_case(wl.CONFIGS["c0"])
