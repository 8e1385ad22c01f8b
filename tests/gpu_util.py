"""Helpers for the GPU parity tests: move a seeded workload to the device, run the C-ABI
entry points through the binding, and evaluate the fp64 oracle on the same inputs."""
import numpy as np
import torch

import workloads as wl

TOL = {wl.BF16: 2e-2, wl.F32: 1e-4}   # max |gpu - ref| / max |ref| per output tensor


def to_dev(a, dtype):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t.to(torch.bfloat16) if dtype == wl.BF16 else t      # inputs are bf16-representable: exact


def dev_inputs(w, d):
    out = {}
    for key, val in d.items():
        out[key] = to_dev(val, w.dtype if key in ("q", "k", "v", "dH") else wl.F32)
    return out


def flat(a):
    """(B, NH, ...) -> (B*NH, ...) float64 for the oracle."""
    a = np.asarray(a, dtype=np.float64)
    return a.reshape((a.shape[0] * a.shape[1],) + a.shape[2:])


def oracle_inputs(d):
    keys = ("q", "k", "v", "i_pre", "f_pre", "C0", "n0", "m0")
    return {k_: (flat(d[k_]) if k_ in d else None) for k_ in keys}


def rel_err(gpu, ref):
    g = gpu.detach().float().cpu().numpy().astype(np.float64).reshape(ref.shape)
    assert np.all(np.isfinite(g)), "non-finite values in GPU output"
    return float(np.max(np.abs(g - ref)) / max(np.max(np.abs(ref)), 1e-30))


def check_fwd(w, d, out, ref, tol=None, state=True, report=None, abs_tol=1e-4):
    tol = TOL[w.dtype] if tol is None else tol
    errs = {"H": rel_err(out["H"], ref["H"])}
    if state:
        errs["Cn"] = rel_err(out["Cn"], ref["Cn"])
    if w.variant == wl.EXP:
        errs["n_out"] = rel_err(out["n_out"], ref["n_out"])
        mo = out["m_out"].float().cpu().numpy().reshape(ref["m_out"].shape)
        errs["m_out_abs"] = float(np.max(np.abs(mo - ref["m_out"]) / np.maximum(1.0, np.abs(ref["m_out"]))))
        if state:
            errs["nn"] = rel_err(out["nn"], ref["nn"])
            mn = out["mn"].float().cpu().numpy().reshape(ref["mn"].shape)
            errs["mn_abs"] = float(np.max(np.abs(mn - ref["mn"]) / np.maximum(1.0, np.abs(ref["mn"]))))
    if report is not None:
        report.update(errs)
    for key, e in errs.items():
        lim = abs_tol if key.endswith("_abs") else tol
        assert e <= lim, (w.name, key, e, errs)
    return errs
