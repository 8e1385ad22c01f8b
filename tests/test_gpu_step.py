"""GPU parity of tfla_mlstm_step (one recurrent step, the generation form) against the fp64
step-by-step oracle (paper Sec. 2.1 / Sec. 4.1): a chain of steps from a random state, and the
hand-over from the chunkwise forward kernel to single steps."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import mlstm_oracle as orc

pytestmark = pytest.mark.gpu


def _dev(a, bf16):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t.to(torch.bfloat16) if bf16 else t


@pytest.mark.parametrize("variant", [wl.EXP, wl.SIG])
@pytest.mark.parametrize("dtype", [wl.BF16, wl.F32])
@pytest.mark.parametrize("dims", [(64, 64), (128, 192), (256, 512), (512, 512), (1024, 1024), (1024, 64)])
def test_step_chain_matches_recurrence(variant, dtype, dims):
    import paper_2503_14376_amd as tfla
    from tests import gpu_util as gu
    dqk, dhv = dims
    K, B, NH = 24, 2, 3
    w = wl.small(variant, dtype, B=B, NH=NH, T=K, dqk=dqk, dhv=dhv, chunk=K, seed=500 + dqk + dhv, init_state=True,
                 backward=False)
    d = wl.make_inputs(w)
    bf = dtype == wl.BF16
    q, k, v = (_dev(d[x], bf) for x in ("q", "k", "v"))
    ip, fp = _dev(d["i_pre"], False), _dev(d["f_pre"], False)
    C, n, m = _dev(d["C0"], False), _dev(d["n0"], False), _dev(d["m0"], False)
    hs = []
    for t in range(K):
        o = tfla.mlstm_step(q[:, :, t].contiguous(), k[:, :, t].contiguous(), v[:, :, t].contiguous(),
                            ip[:, :, t].contiguous(), fp[:, :, t].contiguous(), C, n, m, variant=variant, eps=1e-6,
                            inplace_C=(t % 2 == 1))
        C, n, m = o["C"], o["n"], o["m"]
        hs.append(o["h"].float())
    torch.cuda.synchronize()
    H = torch.stack(hs, dim=2)
    ref = orc.recurrent_fwd(**gu.oracle_inputs(d), variant=variant, eps=1e-6)
    tol = gu.TOL[dtype]
    errs = {"H": gu.rel_err(H, ref["H"]), "C": gu.rel_err(C, ref["Cn"])}
    if variant == wl.EXP:
        errs["n"] = gu.rel_err(n, ref["nn"])
        mn = m.cpu().numpy().reshape(ref["mn"].shape)
        errs["m_abs"] = float(np.max(np.abs(mn - ref["mn"]) / np.maximum(1.0, np.abs(ref["mn"]))))
    else:
        assert float(n.abs().max()) == 0.0 and float(m.abs().max()) == 0.0
    print("step chain", variant, dtype, dims, errs, flush=True)
    for key, e in errs.items():
        assert e <= (1e-4 if key in ("C", "n", "m_abs") else tol), (key, e, errs)


@pytest.mark.parametrize("variant", [wl.EXP, wl.SIG])
def test_forward_then_steps(variant):
    """A prompt through the chunkwise kernel, then single steps from the returned state, equal the
    recurrence over the whole sequence."""
    import paper_2503_14376_amd as tfla
    from tests import gpu_util as gu
    T0, K = 512, 8
    w = wl.small(variant, wl.BF16, B=1, NH=2, T=T0 + K, dqk=128, dhv=256, chunk=128, seed=611, init_state=False,
                 backward=False)
    d = wl.make_inputs(w)
    dev = gu.dev_inputs(w, d)
    head = {k_: v_[:, :, :T0].contiguous() for k_, v_ in dev.items()}
    f = tfla.mlstm_fwd(head["q"], head["k"], head["v"], head["i_pre"], head["f_pre"], chunk=128, variant=variant, eps=1e-6)
    C, n, m = f["Cn"], f["nn"], f["mn"]
    hs = []
    for t in range(T0, T0 + K):
        o = tfla.mlstm_step(dev["q"][:, :, t].contiguous(), dev["k"][:, :, t].contiguous(), dev["v"][:, :, t].contiguous(),
                            dev["i_pre"][:, :, t].contiguous(), dev["f_pre"][:, :, t].contiguous(), C, n, m,
                            variant=variant, eps=1e-6)
        C, n, m = o["C"], o["n"], o["m"]
        hs.append(o["h"].float())
    torch.cuda.synchronize()
    ref = orc.recurrent_fwd(**gu.oracle_inputs(d), variant=variant, eps=1e-6)
    e_h = gu.rel_err(torch.stack(hs, dim=2), ref["H"][:, T0:])
    e_c = gu.rel_err(C, ref["Cn"])
    print("forward then steps", variant, e_h, e_c, flush=True)
    assert e_h <= 2e-2 and e_c <= 2e-2
