"""Helpers for the GPU parity tests: move a seeded workload to the device, run the C-ABI
entry points through the binding, and evaluate the fp64 oracle on the same inputs."""
import numpy as np
import torch

import workloads as wl

TOL = {wl.BF16: 2e-2, wl.F32: 1e-4}   # max |gpu - ref| / max |ref| per output tensor


# moving workloads to the device and to the oracle's layout lives with the input generators
to_dev, dev_inputs, flat, oracle_inputs = wl.to_dev, wl.dev_inputs, wl.flat, wl.oracle_inputs


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
