"""ctypes binding with the same names and argument order as include/tfla_mlstm.h."""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional

EXP, SIG = 0, 1
F32, BF16 = 0, 1
FWD, BWD = 0, 1
NORM_RMS, NORM_LAYER = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "lib", "libtfla_mlstm.so")
_lib = None

EXPORTS = ("tfla_mlstm_fwd", "tfla_mlstm_bwd", "tfla_mlstm_step", "tfla_mlstm_workspace_bytes", "tfla_mlstm_check",
           "tfla_status_string", "tfla_version", "tfla_profile_enable", "tfla_profile_read",
           "tfla_profile_kernels", "tfla_mlstm_layer_fwd", "tfla_mlstm_layer_bwd", "tfla_mlstm_layer_workspace_bytes",
           "tfla_transfer_gain", "tfla_mlstm_layer_step", "tfla_tile_width", "tfla_mlstm_fwd_static",
           "tfla_static_scratch_bytes")


class TflaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed with status %d: %s" % (where, status, status_string(status)))


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads libtfla_mlstm.so; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError("libtfla_mlstm.so is missing at %s: build it with "
                          "`python -m paper_2503_14376_amd.build` (there is no fallback path)" % _LIB_PATH)
    lib = ctypes.CDLL(_LIB_PATH)
    vp, fp, ci, cf, sz = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    lib.tfla_mlstm_fwd.restype = ci
    lib.tfla_mlstm_fwd.argtypes = [vp, vp, vp, fp, fp, fp, fp, fp, ci, ci, ci, ci, ci, ci, ci, ci, cf,
                                   vp, fp, fp, fp, fp, fp, vp, sz, vp]
    lib.tfla_mlstm_fwd_static.restype = ci
    lib.tfla_mlstm_fwd_static.argtypes = [vp, vp, vp, fp, fp, fp, fp, fp, ci, ci, ci, ci, ci, ci, ci, ci, cf,
                                          vp, fp, fp, fp, fp, fp, vp]
    lib.tfla_static_scratch_bytes.restype = sz
    lib.tfla_static_scratch_bytes.argtypes = []
    lib.tfla_mlstm_bwd.restype = ci
    lib.tfla_mlstm_bwd.argtypes = [vp, vp, vp, fp, fp, fp, fp, fp, fp, fp, vp, fp, ci, ci, ci, ci, ci, ci, ci, ci, cf,
                                   vp, vp, vp, fp, fp, fp, vp, sz, vp, sz, vp]
    lib.tfla_mlstm_step.restype = ci
    lib.tfla_mlstm_step.argtypes = [vp, vp, vp, fp, fp, fp, fp, fp, ci, ci, ci, ci, ci, ci, cf, vp, fp, fp, fp, vp]
    lib.tfla_mlstm_layer_fwd.restype = ci
    lib.tfla_mlstm_layer_fwd.argtypes = [vp, vp, vp, fp, fp, vp, fp, fp, fp, fp, fp, ci, ci, ci, ci, ci, ci, ci, ci, cf,
                                         cf, ci, cf, vp, vp, fp, fp, fp, fp, fp, vp, sz, vp]
    lib.tfla_mlstm_layer_bwd.restype = ci
    lib.tfla_mlstm_layer_bwd.argtypes = [vp, vp, vp, fp, fp, vp, fp, fp, fp, fp, fp, vp, fp, fp, vp, fp,
                                         ci, ci, ci, ci, ci, ci, ci, ci, cf, cf, ci, cf,
                                         vp, vp, vp, fp, fp, vp, fp, fp, fp, vp, sz, vp, sz, vp]
    lib.tfla_mlstm_layer_workspace_bytes.restype = sz
    lib.tfla_mlstm_layer_workspace_bytes.argtypes = [ci] * 9
    lib.tfla_mlstm_layer_step.restype = ci
    lib.tfla_mlstm_layer_step.argtypes = [vp, vp, vp, fp, fp, vp, fp, fp, fp, fp, fp, ci, ci, ci, ci, ci, ci, cf, cf, ci, cf,
                                          vp, vp, fp, fp, fp, vp]
    lib.tfla_transfer_gain.restype = ci
    lib.tfla_transfer_gain.argtypes = [vp, vp, ci, ci, ci, ci, ci, ci, cf, fp, fp, vp]
    lib.tfla_mlstm_workspace_bytes.restype = sz
    lib.tfla_mlstm_workspace_bytes.argtypes = [ci] * 9
    lib.tfla_mlstm_check.restype = ci
    lib.tfla_mlstm_check.argtypes = [ci] * 9
    lib.tfla_status_string.restype = ctypes.c_char_p
    lib.tfla_status_string.argtypes = [ci]
    lib.tfla_version.restype = ci
    lib.tfla_profile_enable.restype = ci
    lib.tfla_profile_enable.argtypes = [ci]
    lib.tfla_profile_read.restype = ci
    lib.tfla_profile_read.argtypes = [ci, ctypes.c_char_p, ci, ctypes.POINTER(ctypes.c_double),
                                      ctypes.POINTER(ctypes.c_long)]
    lib.tfla_profile_kernels.restype = ci
    lib.tfla_tile_width.restype = ci
    lib.tfla_tile_width.argtypes = [ci]
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().tfla_status_string(int(status)).decode()


def workspace_bytes(direction, B, NH, T, dqk, dhv, chunk, variant, dtype) -> int:
    return int(load_library().tfla_mlstm_workspace_bytes(direction, B, NH, T, dqk, dhv, chunk, variant, dtype))


def layer_workspace_bytes(direction, B, NH, T, dqk, dhv, chunk, variant, dtype) -> int:
    return int(load_library().tfla_mlstm_layer_workspace_bytes(direction, B, NH, T, dqk, dhv, chunk, variant, dtype))


def check(direction, B, NH, T, dqk, dhv, chunk, variant, dtype) -> int:
    return int(load_library().tfla_mlstm_check(direction, B, NH, T, dqk, dhv, chunk, variant, dtype))


def tile_width(width: int) -> None:
    """Output-column block of the bf16 tiled kernels for tile-size sweeps: 0 = automatic, 64, 128 (256 = automatic)."""
    rc = load_library().tfla_tile_width(int(width))
    if rc != 0:
        raise TflaError(rc, "tfla_tile_width")


def profile_enable(max_launches: int) -> None:
    rc = load_library().tfla_profile_enable(int(max_launches))
    if rc != 0:
        raise TflaError(rc, "tfla_profile_enable")


def profile_read() -> Dict[str, Dict[str, float]]:
    """Per-kernel-family totals since tfla_profile_enable: {name: {ms, launches}}."""
    lib = load_library()
    out = {}
    for kidx in range(lib.tfla_profile_kernels()):
        name = ctypes.create_string_buffer(64)
        ms, n = ctypes.c_double(0.0), ctypes.c_long(0)
        lib.tfla_profile_read(kidx, name, 64, ctypes.byref(ms), ctypes.byref(n))
        out[name.value.decode()] = {"ms": ms.value, "launches": n.value}
    return out


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _torch_dtype(dtype):
    import torch
    return torch.bfloat16 if dtype == BF16 else torch.float32


def _stream_handle(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _want(t, dtype, shape, name):
    if t is None:
        return
    if not t.is_cuda or not t.is_contiguous() or t.dtype != dtype or tuple(t.shape) != tuple(shape):
        raise ValueError("%s must be a contiguous device tensor of dtype %s and shape %s (got %s %s)"
                         % (name, dtype, tuple(shape), t.dtype, tuple(t.shape)))


def mlstm_fwd(q, k, v, i_pre, f_pre, C0=None, n0=None, m0=None, chunk=256, variant=EXP, eps=1e-6,
              return_state=True, workspace=None, stream=None, out: Optional[Dict] = None) -> Dict:
    """tfla_mlstm_fwd on torch device tensors.  q,k: (B,NH,T,dqk); v: (B,NH,T,dhv) in bf16 or
    fp32; gates fp32 (B,NH,T).  Returns a dict with H, Cn, nn, mn, n_out, m_out."""
    import torch
    lib = load_library()
    B, NH, T, dqk = q.shape
    dhv = v.shape[-1]
    dtype = BF16 if q.dtype == torch.bfloat16 else F32
    td, f32 = _torch_dtype(dtype), torch.float32
    _want(q, td, (B, NH, T, dqk), "q"); _want(k, td, (B, NH, T, dqk), "k"); _want(v, td, (B, NH, T, dhv), "v")
    _want(i_pre, f32, (B, NH, T), "i_pre"); _want(f_pre, f32, (B, NH, T), "f_pre")
    _want(C0, f32, (B, NH, dqk, dhv), "C0"); _want(n0, f32, (B, NH, dqk), "n0"); _want(m0, f32, (B, NH), "m0")
    dev = q.device
    o = out if out is not None else {}
    if "H" not in o:
        o["H"] = torch.empty((B, NH, T, dhv), dtype=td, device=dev)
    if return_state and "Cn" not in o:
        o["Cn"] = torch.empty((B, NH, dqk, dhv), dtype=f32, device=dev)
        o["nn"] = torch.empty((B, NH, dqk), dtype=f32, device=dev)
        o["mn"] = torch.empty((B, NH), dtype=f32, device=dev)
    if "n_out" not in o:
        o["n_out"] = torch.empty((B, NH, T), dtype=f32, device=dev)
        o["m_out"] = torch.empty((B, NH, T), dtype=f32, device=dev)
    need = workspace_bytes(FWD, B, NH, T, dqk, dhv, chunk, variant, dtype)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    rc = lib.tfla_mlstm_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(i_pre), _ptr(f_pre), _ptr(C0), _ptr(n0), _ptr(m0),
                            B, NH, T, dqk, dhv, int(chunk), int(variant), dtype, float(eps),
                            _ptr(o["H"]), _ptr(o.get("Cn")), _ptr(o.get("nn")), _ptr(o.get("mn")),
                            _ptr(o["n_out"]), _ptr(o["m_out"]),
                            _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream_handle(stream))
    if rc != 0:
        raise TflaError(rc, "tfla_mlstm_fwd")
    o["workspace"] = workspace
    return o


def static_scratch_bytes() -> int:
    return int(load_library().tfla_static_scratch_bytes())


def mlstm_fwd_static(q, k, v, i_pre, f_pre, C0=None, n0=None, m0=None, chunk=256, variant=EXP, eps=1e-6, stream=None,
                     out: Optional[Dict] = None) -> Dict:
    """tfla_mlstm_fwd_static on torch device tensors: the forward pass on the library's own static scratch memory.
    `out` must hold every output tensor (H, Cn, nn, mn, n_out, m_out; the state and per-step entries may be
    missing = not wanted): this wrapper allocates nothing either."""
    import torch
    lib = load_library()
    B, NH, T, dqk = q.shape
    dhv = v.shape[-1]
    dtype = BF16 if q.dtype == torch.bfloat16 else F32
    td, f32 = _torch_dtype(dtype), torch.float32
    _want(q, td, (B, NH, T, dqk), "q"); _want(k, td, (B, NH, T, dqk), "k"); _want(v, td, (B, NH, T, dhv), "v")
    _want(i_pre, f32, (B, NH, T), "i_pre"); _want(f_pre, f32, (B, NH, T), "f_pre")
    _want(C0, f32, (B, NH, dqk, dhv), "C0"); _want(n0, f32, (B, NH, dqk), "n0"); _want(m0, f32, (B, NH), "m0")
    if out is None or "H" not in out:
        raise ValueError("mlstm_fwd_static writes into caller-provided tensors: pass out={'H': ..., ...}")
    o = out
    _want(o["H"], td, (B, NH, T, dhv), "H"); _want(o.get("Cn"), f32, (B, NH, dqk, dhv), "Cn")
    _want(o.get("nn"), f32, (B, NH, dqk), "nn"); _want(o.get("mn"), f32, (B, NH), "mn")
    _want(o.get("n_out"), f32, (B, NH, T), "n_out"); _want(o.get("m_out"), f32, (B, NH, T), "m_out")
    rc = lib.tfla_mlstm_fwd_static(_ptr(q), _ptr(k), _ptr(v), _ptr(i_pre), _ptr(f_pre), _ptr(C0), _ptr(n0), _ptr(m0),
                                   B, NH, T, dqk, dhv, int(chunk), int(variant), dtype, float(eps),
                                   _ptr(o["H"]), _ptr(o.get("Cn")), _ptr(o.get("nn")), _ptr(o.get("mn")),
                                   _ptr(o.get("n_out")), _ptr(o.get("m_out")), _stream_handle(stream))
    if rc != 0:
        raise TflaError(rc, "tfla_mlstm_fwd_static")
    return o


def mlstm_bwd(q, k, v, i_pre, f_pre, dH, n_out=None, m_out=None, C0=None, n0=None, m0=None, dCn=None,
              chunk=256, variant=EXP, eps=1e-6, want_dC0=True, workspace=None, stream=None,
              out: Optional[Dict] = None, fwd_workspace=None) -> Dict:
    """tfla_mlstm_bwd on torch device tensors.  Returns dq, dk, dv, d_i_pre, d_f_pre, dC0.
    fwd_workspace: the (untouched) workspace tensor of the matching mlstm_fwd call, or None to
    recompute gates and chunk states."""
    import torch
    lib = load_library()
    B, NH, T, dqk = q.shape
    dhv = v.shape[-1]
    dtype = BF16 if q.dtype == torch.bfloat16 else F32
    td, f32 = _torch_dtype(dtype), torch.float32
    _want(q, td, (B, NH, T, dqk), "q"); _want(k, td, (B, NH, T, dqk), "k"); _want(v, td, (B, NH, T, dhv), "v")
    _want(dH, td, (B, NH, T, dhv), "dH")
    _want(i_pre, f32, (B, NH, T), "i_pre"); _want(f_pre, f32, (B, NH, T), "f_pre")
    _want(n_out, f32, (B, NH, T), "n_out"); _want(m_out, f32, (B, NH, T), "m_out")
    _want(C0, f32, (B, NH, dqk, dhv), "C0"); _want(n0, f32, (B, NH, dqk), "n0"); _want(m0, f32, (B, NH), "m0")
    _want(dCn, f32, (B, NH, dqk, dhv), "dCn")
    dev = q.device
    o = out if out is not None else {}
    if "dq" not in o:
        o["dq"] = torch.empty_like(q); o["dk"] = torch.empty_like(k); o["dv"] = torch.empty_like(v)
        o["d_i_pre"] = torch.empty((B, NH, T), dtype=f32, device=dev)
        o["d_f_pre"] = torch.empty((B, NH, T), dtype=f32, device=dev)
    if want_dC0 and "dC0" not in o:
        o["dC0"] = torch.empty((B, NH, dqk, dhv), dtype=f32, device=dev)
    need = workspace_bytes(BWD, B, NH, T, dqk, dhv, chunk, variant, dtype)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    rc = lib.tfla_mlstm_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(i_pre), _ptr(f_pre), _ptr(C0), _ptr(n0), _ptr(m0),
                            _ptr(n_out), _ptr(m_out), _ptr(dH), _ptr(dCn),
                            B, NH, T, dqk, dhv, int(chunk), int(variant), dtype, float(eps),
                            _ptr(o["dq"]), _ptr(o["dk"]), _ptr(o["dv"]), _ptr(o["d_i_pre"]), _ptr(o["d_f_pre"]),
                            _ptr(o.get("dC0")),
                            _ptr(fwd_workspace), 0 if fwd_workspace is None else fwd_workspace.numel(),
                            _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream_handle(stream))
    if rc != 0:
        raise TflaError(rc, "tfla_mlstm_bwd")
    o["workspace"] = workspace
    return o


def mlstm_step(q, k, v, i_pre, f_pre, C, n=None, m=None, variant=EXP, eps=1e-6, stream=None,
               out: Optional[Dict] = None, inplace_C: bool = False) -> Dict:
    """tfla_mlstm_step on torch device tensors.  q, k: (B,NH,dqk); v: (B,NH,dhv); i_pre, f_pre: (B,NH);
    C: (B,NH,dqk,dhv) fp32, n: (B,NH,dqk), m: (B,NH).  Returns h and the new state C, n, m."""
    import torch
    lib = load_library()
    B, NH, dqk = q.shape
    dhv = v.shape[-1]
    dtype = BF16 if q.dtype == torch.bfloat16 else F32
    td, f32 = _torch_dtype(dtype), torch.float32
    _want(q, td, (B, NH, dqk), "q"); _want(k, td, (B, NH, dqk), "k"); _want(v, td, (B, NH, dhv), "v")
    _want(i_pre, f32, (B, NH), "i_pre"); _want(f_pre, f32, (B, NH), "f_pre")
    _want(C, f32, (B, NH, dqk, dhv), "C"); _want(n, f32, (B, NH, dqk), "n"); _want(m, f32, (B, NH), "m")
    dev = q.device
    o = out if out is not None else {}
    if "h" not in o:
        o["h"] = torch.empty((B, NH, dhv), dtype=td, device=dev)
    if "C" not in o:
        o["C"] = C if inplace_C else torch.empty_like(C)
    if "n" not in o:
        o["n"] = torch.empty((B, NH, dqk), dtype=f32, device=dev)
        o["m"] = torch.empty((B, NH), dtype=f32, device=dev)
    rc = lib.tfla_mlstm_step(_ptr(q), _ptr(k), _ptr(v), _ptr(i_pre), _ptr(f_pre), _ptr(C), _ptr(n), _ptr(m),
                             B, NH, dqk, dhv, int(variant), dtype, float(eps),
                             _ptr(o["h"]), _ptr(o["C"]), _ptr(o["n"]), _ptr(o["m"]), _stream_handle(stream))
    if rc != 0:
        raise TflaError(rc, "tfla_mlstm_step")
    return o


def mlstm_layer_fwd(q, k, v, i_pre, f_pre, o_pre=None, gamma=None, beta=None, C0=None, n0=None, m0=None, chunk=256,
                    variant=EXP, eps=1e-6, gate_softcap=0.0, norm_kind=NORM_RMS, norm_eps=1e-6, return_state=True,
                    workspace=None, stream=None, out: Optional[Dict] = None) -> Dict:
    """tfla_mlstm_layer_fwd on torch device tensors: soft-capped gates, cell, multi-head norm, output gate.
    o_pre: (B,NH,T,dhv) like v or None; gamma, beta: (NH,dhv) fp32 or None.  Returns Y, H (cell output), the
    final state, n_out, m_out and the workspace."""
    import torch
    lib = load_library()
    B, NH, T, dqk = q.shape
    dhv = v.shape[-1]
    dtype = BF16 if q.dtype == torch.bfloat16 else F32
    td, f32 = _torch_dtype(dtype), torch.float32
    _want(q, td, (B, NH, T, dqk), "q"); _want(k, td, (B, NH, T, dqk), "k"); _want(v, td, (B, NH, T, dhv), "v")
    _want(i_pre, f32, (B, NH, T), "i_pre"); _want(f_pre, f32, (B, NH, T), "f_pre")
    _want(o_pre, td, (B, NH, T, dhv), "o_pre"); _want(gamma, f32, (NH, dhv), "gamma"); _want(beta, f32, (NH, dhv), "beta")
    _want(C0, f32, (B, NH, dqk, dhv), "C0"); _want(n0, f32, (B, NH, dqk), "n0"); _want(m0, f32, (B, NH), "m0")
    dev = q.device
    o = out if out is not None else {}
    if "Y" not in o:
        o["Y"] = torch.empty((B, NH, T, dhv), dtype=td, device=dev)
        o["H"] = torch.empty((B, NH, T, dhv), dtype=td, device=dev)
    if return_state and "Cn" not in o:
        o["Cn"] = torch.empty((B, NH, dqk, dhv), dtype=f32, device=dev)
        o["nn"] = torch.empty((B, NH, dqk), dtype=f32, device=dev)
        o["mn"] = torch.empty((B, NH), dtype=f32, device=dev)
    if "n_out" not in o:
        o["n_out"] = torch.empty((B, NH, T), dtype=f32, device=dev)
        o["m_out"] = torch.empty((B, NH, T), dtype=f32, device=dev)
    need = layer_workspace_bytes(FWD, B, NH, T, dqk, dhv, chunk, variant, dtype)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    rc = lib.tfla_mlstm_layer_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(i_pre), _ptr(f_pre), _ptr(o_pre), _ptr(gamma), _ptr(beta),
                                  _ptr(C0), _ptr(n0), _ptr(m0), B, NH, T, dqk, dhv, int(chunk), int(variant), dtype,
                                  float(eps), float(gate_softcap), int(norm_kind), float(norm_eps),
                                  _ptr(o["Y"]), _ptr(o["H"]), _ptr(o.get("Cn")), _ptr(o.get("nn")), _ptr(o.get("mn")),
                                  _ptr(o["n_out"]), _ptr(o["m_out"]),
                                  _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream_handle(stream))
    if rc != 0:
        raise TflaError(rc, "tfla_mlstm_layer_fwd")
    o["workspace"] = workspace
    return o


def mlstm_layer_bwd(q, k, v, i_pre, f_pre, H, dY, o_pre=None, gamma=None, beta=None, n_out=None, m_out=None, C0=None,
                    n0=None, m0=None, dCn=None, chunk=256, variant=EXP, eps=1e-6, gate_softcap=0.0, norm_kind=NORM_RMS,
                    norm_eps=1e-6, want_dC0=True, workspace=None, stream=None, out: Optional[Dict] = None,
                    fwd_workspace=None) -> Dict:
    """tfla_mlstm_layer_bwd on torch device tensors.  Returns dq, dk, dv, d_i_pre, d_f_pre, do_pre (if o_pre is
    given), dgamma, dbeta, dC0."""
    import torch
    lib = load_library()
    B, NH, T, dqk = q.shape
    dhv = v.shape[-1]
    dtype = BF16 if q.dtype == torch.bfloat16 else F32
    td, f32 = _torch_dtype(dtype), torch.float32
    _want(q, td, (B, NH, T, dqk), "q"); _want(k, td, (B, NH, T, dqk), "k"); _want(v, td, (B, NH, T, dhv), "v")
    _want(H, td, (B, NH, T, dhv), "H"); _want(dY, td, (B, NH, T, dhv), "dY"); _want(o_pre, td, (B, NH, T, dhv), "o_pre")
    _want(gamma, f32, (NH, dhv), "gamma"); _want(beta, f32, (NH, dhv), "beta")
    _want(i_pre, f32, (B, NH, T), "i_pre"); _want(f_pre, f32, (B, NH, T), "f_pre")
    _want(n_out, f32, (B, NH, T), "n_out"); _want(m_out, f32, (B, NH, T), "m_out")
    _want(C0, f32, (B, NH, dqk, dhv), "C0"); _want(n0, f32, (B, NH, dqk), "n0"); _want(m0, f32, (B, NH), "m0")
    _want(dCn, f32, (B, NH, dqk, dhv), "dCn")
    dev = q.device
    o = out if out is not None else {}
    if "dq" not in o:
        o["dq"] = torch.empty_like(q); o["dk"] = torch.empty_like(k); o["dv"] = torch.empty_like(v)
        o["d_i_pre"] = torch.empty((B, NH, T), dtype=f32, device=dev)
        o["d_f_pre"] = torch.empty((B, NH, T), dtype=f32, device=dev)
        o["dgamma"] = torch.empty((NH, dhv), dtype=f32, device=dev)
        o["dbeta"] = torch.empty((NH, dhv), dtype=f32, device=dev)
        if o_pre is not None:
            o["do_pre"] = torch.empty_like(o_pre)
    if want_dC0 and "dC0" not in o:
        o["dC0"] = torch.empty((B, NH, dqk, dhv), dtype=f32, device=dev)
    need = layer_workspace_bytes(BWD, B, NH, T, dqk, dhv, chunk, variant, dtype)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    rc = lib.tfla_mlstm_layer_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(i_pre), _ptr(f_pre), _ptr(o_pre), _ptr(gamma), _ptr(beta),
                                  _ptr(C0), _ptr(n0), _ptr(m0), _ptr(H), _ptr(n_out), _ptr(m_out), _ptr(dY), _ptr(dCn),
                                  B, NH, T, dqk, dhv, int(chunk), int(variant), dtype, float(eps), float(gate_softcap),
                                  int(norm_kind), float(norm_eps),
                                  _ptr(o["dq"]), _ptr(o["dk"]), _ptr(o["dv"]), _ptr(o["d_i_pre"]), _ptr(o["d_f_pre"]),
                                  _ptr(o.get("do_pre")), _ptr(o.get("dgamma")), _ptr(o.get("dbeta")), _ptr(o.get("dC0")),
                                  _ptr(fwd_workspace), 0 if fwd_workspace is None else fwd_workspace.numel(),
                                  _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream_handle(stream))
    if rc != 0:
        raise TflaError(rc, "tfla_mlstm_layer_bwd")
    o["workspace"] = workspace
    return o


def mlstm_layer_step(q, k, v, i_pre, f_pre, C, n=None, m=None, o_pre=None, gamma=None, beta=None, variant=EXP, eps=1e-6,
                     gate_softcap=0.0, norm_kind=NORM_RMS, norm_eps=1e-6, stream=None, out: Optional[Dict] = None,
                     inplace_C: bool = False) -> Dict:
    """tfla_mlstm_layer_step on torch device tensors: mlstm_step with soft-capped gates, then norm and output gate.
    o_pre: (B,NH,dhv) like v or None.  Returns y, h (cell output) and the new state C, n, m."""
    import torch
    lib = load_library()
    B, NH, dqk = q.shape
    dhv = v.shape[-1]
    dtype = BF16 if q.dtype == torch.bfloat16 else F32
    td, f32 = _torch_dtype(dtype), torch.float32
    _want(q, td, (B, NH, dqk), "q"); _want(k, td, (B, NH, dqk), "k"); _want(v, td, (B, NH, dhv), "v")
    _want(o_pre, td, (B, NH, dhv), "o_pre"); _want(gamma, f32, (NH, dhv), "gamma"); _want(beta, f32, (NH, dhv), "beta")
    _want(i_pre, f32, (B, NH), "i_pre"); _want(f_pre, f32, (B, NH), "f_pre")
    _want(C, f32, (B, NH, dqk, dhv), "C"); _want(n, f32, (B, NH, dqk), "n"); _want(m, f32, (B, NH), "m")
    dev = q.device
    o = out if out is not None else {}
    if "y" not in o:
        o["y"] = torch.empty((B, NH, dhv), dtype=td, device=dev)
        o["h"] = torch.empty((B, NH, dhv), dtype=td, device=dev)
    if "C" not in o:
        o["C"] = C if inplace_C else torch.empty_like(C)
    if "n" not in o:
        o["n"] = torch.empty((B, NH, dqk), dtype=f32, device=dev)
        o["m"] = torch.empty((B, NH), dtype=f32, device=dev)
    rc = lib.tfla_mlstm_layer_step(_ptr(q), _ptr(k), _ptr(v), _ptr(i_pre), _ptr(f_pre), _ptr(o_pre), _ptr(gamma), _ptr(beta),
                                   _ptr(C), _ptr(n), _ptr(m), B, NH, dqk, dhv, int(variant), dtype, float(eps),
                                   float(gate_softcap), int(norm_kind), float(norm_eps), _ptr(o["y"]), _ptr(o["h"]),
                                   _ptr(o["C"]), _ptr(o["n"]), _ptr(o["m"]), _stream_handle(stream))
    if rc != 0:
        raise TflaError(rc, "tfla_mlstm_layer_step")
    return o


def transfer_gain(h, v, norm_kind=NORM_RMS, norm_eps=1e-6, stream=None):
    """tfla_transfer_gain on torch device tensors h, v (B,NH,T,dhv).  Returns (g_before, g_after), each (B,NH) fp32."""
    import torch
    lib = load_library()
    B, NH, T, dhv = h.shape
    dtype = BF16 if h.dtype == torch.bfloat16 else F32
    td = _torch_dtype(dtype)
    _want(h, td, (B, NH, T, dhv), "h"); _want(v, td, (B, NH, T, dhv), "v")
    gb = torch.empty((B, NH), dtype=torch.float32, device=h.device)
    ga = torch.empty((B, NH), dtype=torch.float32, device=h.device)
    rc = lib.tfla_transfer_gain(_ptr(h), _ptr(v), B, NH, T, dhv, dtype, int(norm_kind), float(norm_eps), _ptr(gb), _ptr(ga),
                                _stream_handle(stream))
    if rc != 0:
        raise TflaError(rc, "tfla_transfer_gain")
    return gb, ga
