"""The two entry points under HIP graph capture: the library allocates nothing, never synchronises and
records no memset nodes, so a captured forward + backward step must replay to exactly the eager
result, every time, also with eager work and synchronisations between the replays."""
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("variant", [wl.EXP, wl.SIG])
def test_graph_replay_matches_eager(variant):
    import paper_2503_14376_amd as tfla
    from tests import gpu_util as gu
    w = wl.small(variant, wl.BF16, B=1, NH=2, T=1024, dqk=128, dhv=256, chunk=256, seed=77, init_state=False)
    dev = gu.dev_inputs(w, wl.make_inputs(w))
    w2 = wl.small(variant, wl.BF16, B=1, NH=2, T=1024, dqk=128, dhv=256, chunk=256, seed=78, init_state=False)
    dev2 = gu.dev_inputs(w2, wl.make_inputs(w2))
    ws_f = torch.empty(tfla.workspace_bytes(0, 1, 2, 1024, 128, 256, 256, variant, wl.BF16), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(tfla.workspace_bytes(1, 1, 2, 1024, 128, 256, 256, variant, wl.BF16), dtype=torch.uint8, device="cuda")

    def step(d, fo, bo, wf, wb):
        tfla.mlstm_fwd(d["q"], d["k"], d["v"], d["i_pre"], d["f_pre"], chunk=256, variant=variant, eps=1e-6,
                       workspace=wf, out=fo)
        tfla.mlstm_bwd(d["q"], d["k"], d["v"], d["i_pre"], d["f_pre"], d["dH"], fo["n_out"], fo["m_out"], chunk=256,
                       variant=variant, eps=1e-6, workspace=wb, out=bo, fwd_workspace=wf)

    keys_f, keys_b = ("H", "Cn", "n_out", "m_out"), ("dq", "dk", "dv", "d_i_pre", "d_f_pre", "dC0")

    def snapshot(fo, bo):
        return [fo[k_].clone() for k_ in keys_f] + [bo[k_].clone() for k_ in keys_b]

    def eager(d):
        fo, bo = {}, {}
        step(d, fo, bo, torch.empty_like(ws_f), torch.empty_like(ws_b))
        torch.cuda.synchronize()
        return snapshot(fo, bo)

    ref1, ref2 = eager(dev), eager(dev2)

    # static buffers of the graph
    g_in = {k_: v_.clone() for k_, v_ in dev.items()}
    fo, bo = {}, {}
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(g_in, fo, bo, ws_f, ws_b)          # allocates the outputs before the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(g_in, fo, bo, ws_f, ws_b)

    def check(ref):
        torch.cuda.synchronize()
        for got, want in zip(snapshot(fo, bo), ref):
            assert torch.equal(got, want)

    for rep in range(4):
        src, ref = (dev, ref1) if rep % 2 == 0 else (dev2, ref2)
        for k_ in g_in:
            g_in[k_].copy_(src[k_])
        for k_ in keys_f:
            fo[k_].zero_()
        for k_ in keys_b:
            bo[k_].zero_()
        graph.replay()
        check(ref)
        eager(dev2 if rep % 2 == 0 else dev)     # eager work of the same library between the replays


def test_graph_replay_layer_with_ragged_length():
    """The layer entry points with a sequence length that does not fill its last chunk (padding copies, gate soft-cap,
    norm, parameter-gradient reduction): captured once, replayed with changing inputs, bit-equal to eager."""
    import paper_2503_14376_amd as tfla
    from tests.test_gpu_layer import _dev
    B, NH, T, dqk, dhv, chunk, variant = 2, 2, 600, 64, 128, 256, wl.EXP
    mk = lambda seed: wl.small(variant, wl.BF16, B=B, NH=NH, T=T, dqk=dqk, dhv=dhv, chunk=chunk, seed=seed, init_state=False)
    devs = [_dev(mk(s), wl.make_layer_inputs(mk(s), None, 2.0)) for s in (91, 92)]
    ws_f = torch.empty(tfla.layer_workspace_bytes(0, B, NH, T, dqk, dhv, chunk, variant, wl.BF16), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(tfla.layer_workspace_bytes(1, B, NH, T, dqk, dhv, chunk, variant, wl.BF16), dtype=torch.uint8, device="cuda")
    kw = dict(chunk=chunk, variant=variant, eps=1e-6, gate_softcap=15.0, norm_kind=tfla.NORM_LAYER, norm_eps=1e-6)

    def step(d, fo, bo, wf, wb):
        tfla.mlstm_layer_fwd(d["q"], d["k"], d["v"], d["i_pre"], d["f_pre"], d["o_pre"], d["gamma"], d["beta"],
                             workspace=wf, out=fo, **kw)
        tfla.mlstm_layer_bwd(d["q"], d["k"], d["v"], d["i_pre"], d["f_pre"], fo["H"], d["dH"], d["o_pre"], d["gamma"],
                             d["beta"], fo["n_out"], fo["m_out"], workspace=wb, out=bo, fwd_workspace=wf, **kw)

    keys_f = ("Y", "H", "Cn", "n_out", "m_out")
    keys_b = ("dq", "dk", "dv", "d_i_pre", "d_f_pre", "do_pre", "dgamma", "dbeta", "dC0")
    snapshot = lambda fo, bo: [fo[k_].clone() for k_ in keys_f] + [bo[k_].clone() for k_ in keys_b]

    def eager(d):
        fo, bo = {}, {}
        step(d, fo, bo, torch.empty_like(ws_f), torch.empty_like(ws_b))
        torch.cuda.synchronize()
        return snapshot(fo, bo)

    refs = [eager(d) for d in devs]
    g_in = {k_: v_.clone() for k_, v_ in devs[0].items()}
    fo, bo = {}, {}
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(g_in, fo, bo, ws_f, ws_b)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(g_in, fo, bo, ws_f, ws_b)
    for rep in range(4):
        for k_ in g_in:
            g_in[k_].copy_(devs[rep % 2][k_])
        for k_ in keys_f:
            fo[k_].zero_()
        for k_ in keys_b:
            bo[k_].zero_()
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip(snapshot(fo, bo), refs[rep % 2]):
            assert torch.equal(got, want)
        eager(devs[(rep + 1) % 2])
