"""Thin Python binding of libgsa: same entry points as include/gsa.h, torch tensors in.

Argument marshalling only -- every step of the operator runs in the HIP kernels.
PyTorch supplies device memory and the current stream, nothing else.
"""
import ctypes
from typing import Optional

import torch

from . import _lib

GSA_F32, GSA_BF16 = 0, 1
_DTYPES = {torch.float32: GSA_F32, torch.bfloat16: GSA_BF16}


class GsaError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = _lib.load().gsa_status_string(code).decode()
        super().__init__("%s failed: %s (status %d)" % (where, msg, code))


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _check(t, name, dtype=None, shape=None, optional=False):
    if t is None:
        if optional:
            return
        raise ValueError("%s is required" % name)
    if not t.is_cuda:
        raise ValueError("%s must live on the GPU" % name)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if dtype is not None and t.dtype != dtype:
        raise ValueError("%s must be %s, got %s" % (name, dtype, t.dtype))
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("%s must have shape %s, got %s" % (name, tuple(shape), tuple(t.shape)))


def _stream(t: torch.Tensor):
    return ctypes.c_void_p(torch.cuda.current_stream(t.device).cuda_stream)


def make_problem(q, v, g, scale=1.0, cu_seqlens=None, keep_states=False):
    B, T, H, d_k = q.shape
    d_v, m = v.shape[-1], g.shape[-1]
    if q.dtype not in _DTYPES:
        raise ValueError("q,k,v must be float32 or bfloat16")
    p = _lib.GsaProblem()
    p.B, p.T, p.H, p.d_k, p.d_v, p.m = B, T, H, d_k, d_v, m
    p.dtype = _DTYPES[q.dtype]
    p.scale = float(scale)
    p.keep_states = int(bool(keep_states))
    if cu_seqlens is not None:
        _check(cu_seqlens, "cu_seqlens", torch.int32)
        p.cu_seqlens = cu_seqlens.data_ptr()
        p.n_seqs = cu_seqlens.numel() - 1
    else:
        p.cu_seqlens = None
        p.n_seqs = B
    return p


def gsa_workspace_bytes(problem, want_bwd: bool) -> int:
    n = ctypes.c_size_t(0)
    rc = _lib.load().gsa_workspace_bytes(ctypes.byref(problem), int(bool(want_bwd)), ctypes.byref(n))
    if rc != 0:
        raise GsaError(rc, "gsa_workspace_bytes")
    return int(n.value)


def alloc_workspace(problem, want_bwd: bool, device) -> torch.Tensor:
    n = gsa_workspace_bytes(problem, want_bwd)
    return torch.empty(max(n, 256), dtype=torch.uint8, device=device)


READOUTS = {"softmax": 0, "identity": 1, "swish": 2, "relu": 3, "relu2": 4}
FEATURE_MAPS = {"none": 0, "swish": 1}


def gsa_fwd(q, k, v, g, K0=None, V0=None, scale=1.0, cu_seqlens=None, save_z=True, final_state=False,
            workspace=None, s=None, readout="softmax", gate_tau=0.0, feature_map="none", keep_states=False):
    """Returns (o, z_saved or None, KT or None, VT or None).  keep_states: leave the per-chunk memories in
    `workspace` (then required, of the backward's size) for a gsa_bwd call with keep_states.  With s (write intensities [B,T,H,m] fp32),
    a readout other than "softmax", gate_tau > 0 (g holds gate logits, log gate = logsigmoid(g)/gate_tau)
    or feature_map "swish" (q, k, v hold raw projections, the kernels apply x*sigmoid(x) to them) the call
    goes through gsa_fwd_ex."""
    B, T, H, d_k = q.shape
    d_v, m = v.shape[-1], g.shape[-1]
    p = make_problem(q, v, g, scale, cu_seqlens, keep_states)
    n = p.n_seqs
    _check(q, "q", q.dtype, (B, T, H, d_k)); _check(k, "k", q.dtype, (B, T, H, d_k))
    _check(v, "v", q.dtype, (B, T, H, d_v)); _check(g, "g", torch.float32, (B, T, H, m))
    _check(K0, "K0", torch.float32, (n, H, m, d_k), optional=True)
    _check(V0, "V0", torch.float32, (n, H, m, d_v), optional=True)
    if workspace is None:
        if keep_states:
            raise ValueError("keep_states: pass the workspace that the backward call will be given")
        workspace = alloc_workspace(p, False, q.device)
    o = torch.empty_like(v)
    z = torch.empty((B, T, H, m), dtype=torch.float32, device=q.device) if save_z else None
    KT = torch.empty((n, H, m, d_k), dtype=torch.float32, device=q.device) if final_state else None
    VT = torch.empty((n, H, m, d_v), dtype=torch.float32, device=q.device) if final_state else None
    if s is not None or readout != "softmax" or gate_tau or feature_map != "none":
        _check(s, "s", torch.float32, (B, T, H, m), optional=True)
        rc = _lib.load().gsa_fwd_ex(ctypes.byref(p), READOUTS[readout], float(gate_tau), FEATURE_MAPS[feature_map],
                                    _ptr(q), _ptr(k), _ptr(v), _ptr(g), _ptr(s), _ptr(K0), _ptr(V0), _ptr(o), _ptr(z),
                                    _ptr(KT), _ptr(VT), _ptr(workspace), workspace.numel(), _stream(q))
        if rc != 0:
            raise GsaError(rc, "gsa_fwd_ex")
        return o, z, KT, VT
    rc = _lib.load().gsa_fwd(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(g), _ptr(K0), _ptr(V0),
                             _ptr(o), _ptr(z), _ptr(KT), _ptr(VT), _ptr(workspace), workspace.numel(),
                             _stream(q))
    if rc != 0:
        raise GsaError(rc, "gsa_fwd")
    return o, z, KT, VT


def gsa_fwd_act(q, k, v, g, K0=None, V0=None, scale=1.0, cu_seqlens=None, save_z=True, final_state=False,
                workspace=None, s=None, readout="softmax", gate_tau=0.0, feature_map="none", want_o=True,
                keep_states=False):
    """gsa_fwd_act of the C ABI: the forward with the layer's output epilogue fused in.  Returns
    (o or None, act, act_ssq, z_saved or None, KT or None, VT or None) with act = Swish(o) and act_ssq
    [B,T,H,ceil(d_v/slice)] the per-slice sums of squares of act."""
    B, T, H, d_k = q.shape
    d_v, m = v.shape[-1], g.shape[-1]
    p = make_problem(q, v, g, scale, cu_seqlens, keep_states)
    n = p.n_seqs
    _check(q, "q", q.dtype, (B, T, H, d_k)); _check(k, "k", q.dtype, (B, T, H, d_k))
    _check(v, "v", q.dtype, (B, T, H, d_v)); _check(g, "g", torch.float32, (B, T, H, m))
    _check(K0, "K0", torch.float32, (n, H, m, d_k), optional=True)
    _check(V0, "V0", torch.float32, (n, H, m, d_v), optional=True)
    _check(s, "s", torch.float32, (B, T, H, m), optional=True)
    if workspace is None:
        if keep_states:
            raise ValueError("keep_states: pass the workspace that the backward call will be given")
        workspace = alloc_workspace(p, False, q.device)
    slice_cols = _lib.load().gsa_act_slice_cols(p.dtype)
    o = torch.empty_like(v) if want_o else None
    act = torch.empty_like(v)
    ssq = torch.empty((B, T, H, (d_v + slice_cols - 1) // slice_cols), dtype=torch.float32, device=q.device)
    z = torch.empty((B, T, H, m), dtype=torch.float32, device=q.device) if save_z else None
    KT = torch.empty((n, H, m, d_k), dtype=torch.float32, device=q.device) if final_state else None
    VT = torch.empty((n, H, m, d_v), dtype=torch.float32, device=q.device) if final_state else None
    rc = _lib.load().gsa_fwd_act(ctypes.byref(p), READOUTS[readout], float(gate_tau), FEATURE_MAPS[feature_map],
                                 _ptr(q), _ptr(k), _ptr(v), _ptr(g), _ptr(s), _ptr(K0), _ptr(V0), _ptr(o), _ptr(act),
                                 _ptr(ssq), _ptr(z), _ptr(KT), _ptr(VT), _ptr(workspace), workspace.numel(),
                                 _stream(q))
    if rc != 0:
        raise GsaError(rc, "gsa_fwd_act")
    return o, act, ssq, z, KT, VT


def gsa_bwd(q, k, v, g, z_saved, dO, K0=None, V0=None, dKT=None, dVT=None, scale=1.0, cu_seqlens=None,
            initial_state_grad=False, workspace=None, s=None, readout="softmax", gate_tau=0.0,
            feature_map="none", keep_states=False):
    """Returns (dq, dk, dv, dg, dK0 or None, dV0 or None), plus ds as a seventh item when s is given
    (gsa_bwd_ex; dg is then the gradient through the decay alone).  keep_states: `workspace` is the one the
    forward call with keep_states filled for the same inputs; the per-chunk memories are not recomputed."""
    B, T, H, d_k = q.shape
    d_v, m = v.shape[-1], g.shape[-1]
    p = make_problem(q, v, g, scale, cu_seqlens, keep_states)
    n = p.n_seqs
    _check(q, "q", q.dtype, (B, T, H, d_k)); _check(k, "k", q.dtype, (B, T, H, d_k))
    _check(v, "v", q.dtype, (B, T, H, d_v)); _check(g, "g", torch.float32, (B, T, H, m))
    _check(z_saved, "z_saved", torch.float32, (B, T, H, m)); _check(dO, "dO", q.dtype, (B, T, H, d_v))
    for t, nm, d in ((K0, "K0", d_k), (V0, "V0", d_v), (dKT, "dKT", d_k), (dVT, "dVT", d_v)):
        _check(t, nm, torch.float32, (n, H, m, d), optional=True)
    if workspace is None:
        if keep_states:
            raise ValueError("keep_states: pass the workspace the forward call filled")
        workspace = alloc_workspace(p, True, q.device)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    dg = torch.empty_like(g)
    dK0 = torch.empty((n, H, m, d_k), dtype=torch.float32, device=q.device) if initial_state_grad else None
    dV0 = torch.empty((n, H, m, d_v), dtype=torch.float32, device=q.device) if initial_state_grad else None
    if s is not None or readout != "softmax" or gate_tau or feature_map != "none":
        _check(s, "s", torch.float32, (B, T, H, m), optional=True)
        ds = None if s is None else torch.empty_like(g)
        rc = _lib.load().gsa_bwd_ex(ctypes.byref(p), READOUTS[readout], float(gate_tau), FEATURE_MAPS[feature_map],
                                    _ptr(q), _ptr(k), _ptr(v), _ptr(g), _ptr(s), _ptr(K0), _ptr(V0), _ptr(z_saved),
                                    _ptr(dO), _ptr(dKT), _ptr(dVT), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(dg), _ptr(ds),
                                    _ptr(dK0), _ptr(dV0), _ptr(workspace), workspace.numel(), _stream(q))
        if rc != 0:
            raise GsaError(rc, "gsa_bwd_ex")
        return (dq, dk, dv, dg, dK0, dV0) if s is None else (dq, dk, dv, dg, dK0, dV0, ds)
    rc = _lib.load().gsa_bwd(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(g), _ptr(K0), _ptr(V0),
                             _ptr(z_saved), _ptr(dO), _ptr(dKT), _ptr(dVT), _ptr(dq), _ptr(dk), _ptr(dv),
                             _ptr(dg), _ptr(dK0), _ptr(dV0), _ptr(workspace), workspace.numel(), _stream(q))
    if rc != 0:
        raise GsaError(rc, "gsa_bwd")
    return dq, dk, dv, dg, dK0, dV0


def gsa_decode_workspace_bytes(B, H, d_k, d_v, m) -> int:
    n = ctypes.c_size_t(0)
    rc = _lib.load().gsa_decode_workspace_bytes(B, H, d_k, d_v, m, ctypes.byref(n))
    if rc != 0:
        raise GsaError(rc, "gsa_decode_workspace_bytes")
    return int(n.value)


def alloc_decode_workspace(B, H, d_k, d_v, m, device) -> torch.Tensor:
    return torch.empty(max(gsa_decode_workspace_bytes(B, H, d_k, d_v, m), 256), dtype=torch.uint8, device=device)


def gsa_decode_step(q, k, v, g, K_state, V_state, scale=1.0, out=None, workspace=None, s=None, readout="softmax",
                    gate_tau=0.0, feature_map="none"):
    """q,k [B,H,d_k], v [B,H,d_v], g [B,H,m]; K_state,V_state fp32 [B,H,m,d], updated in place.
    With a workspace (alloc_decode_workspace) the call goes through gsa_decode_step_ws, which spreads
    each memory over several workgroups.  With s ([B,H,m] fp32 write intensities), a readout other than
    "softmax", gate_tau > 0 or feature_map "swish" it goes through gsa_decode_step_ex.  Returns o [B,H,d_v]."""
    B, H, d_k = q.shape
    d_v, m = v.shape[-1], g.shape[-1]
    if q.dtype not in _DTYPES:
        raise ValueError("q,k,v must be float32 or bfloat16")
    _check(q, "q", q.dtype, (B, H, d_k)); _check(k, "k", q.dtype, (B, H, d_k))
    _check(v, "v", q.dtype, (B, H, d_v)); _check(g, "g", torch.float32, (B, H, m))
    _check(K_state, "K_state", torch.float32, (B, H, m, d_k))
    _check(V_state, "V_state", torch.float32, (B, H, m, d_v))
    o = torch.empty_like(v) if out is None else out
    _check(o, "out", q.dtype, (B, H, d_v))
    if s is not None or readout != "softmax" or gate_tau or feature_map != "none":
        _check(s, "s", torch.float32, (B, H, m), optional=True)
        rc = _lib.load().gsa_decode_step_ex(B, H, d_k, d_v, m, _DTYPES[q.dtype], float(scale), READOUTS[readout],
                                            float(gate_tau), FEATURE_MAPS[feature_map],
                                            _ptr(q), _ptr(k), _ptr(v), _ptr(g), _ptr(s), _ptr(K_state),
                                            _ptr(V_state), _ptr(o), _ptr(workspace),
                                            0 if workspace is None else workspace.numel(), _stream(q))
        if rc != 0:
            raise GsaError(rc, "gsa_decode_step_ex")
        return o
    if workspace is not None:
        rc = _lib.load().gsa_decode_step_ws(B, H, d_k, d_v, m, _DTYPES[q.dtype], float(scale), _ptr(q), _ptr(k),
                                            _ptr(v), _ptr(g), _ptr(K_state), _ptr(V_state), _ptr(o),
                                            _ptr(workspace), workspace.numel(), _stream(q))
        if rc != 0:
            raise GsaError(rc, "gsa_decode_step_ws")
        return o
    rc = _lib.load().gsa_decode_step(B, H, d_k, d_v, m, _DTYPES[q.dtype], float(scale), _ptr(q), _ptr(k),
                                     _ptr(v), _ptr(g), _ptr(K_state), _ptr(V_state), _ptr(o), _stream(q))
    if rc != 0:
        raise GsaError(rc, "gsa_decode_step")
    return o


def gsa_decode_step_static(q, k, v, g, K_state, V_state, out, scale=1.0):
    """gsa_decode_step_static of the C ABI: the decode step for callers that cannot allocate (the split
    form's scratch is an array inside the library).  `out` [B,H,d_v] is required: nothing is allocated
    here either.  Raises GsaError (workspace) when the problem exceeds the built-in scratch."""
    B, H, d_k = q.shape
    d_v, m = v.shape[-1], g.shape[-1]
    if q.dtype not in _DTYPES:
        raise ValueError("q,k,v must be float32 or bfloat16")
    _check(q, "q", q.dtype, (B, H, d_k)); _check(k, "k", q.dtype, (B, H, d_k))
    _check(v, "v", q.dtype, (B, H, d_v)); _check(g, "g", torch.float32, (B, H, m))
    _check(K_state, "K_state", torch.float32, (B, H, m, d_k))
    _check(V_state, "V_state", torch.float32, (B, H, m, d_v))
    _check(out, "out", q.dtype, (B, H, d_v))
    rc = _lib.load().gsa_decode_step_static(B, H, d_k, d_v, m, _DTYPES[q.dtype], float(scale), _ptr(q), _ptr(k),
                                            _ptr(v), _ptr(g), _ptr(K_state), _ptr(V_state), _ptr(out), _stream(q))
    if rc != 0:
        raise GsaError(rc, "gsa_decode_step_static")
    return out


def gsa_profile_enable(on: bool) -> None:
    _lib.load().gsa_profile_enable(int(bool(on)))


def gsa_profile_reset() -> None:
    _lib.load().gsa_profile_reset()


def gsa_profile_copy(dst, src) -> None:
    """Plain device copy src -> dst with the library's probe kernel (same byte count read and written)."""
    if dst.device != src.device or not dst.is_cuda or not dst.is_contiguous() or not src.is_contiguous():
        raise ValueError("dst and src must be contiguous tensors on the same GPU")
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("dst and src must hold the same number of bytes")
    rc = _lib.load().gsa_profile_copy(_ptr(dst), _ptr(src), nbytes, _stream(src))
    if rc != 0:
        raise GsaError(rc, "gsa_profile_copy")


def gsa_profile_read():
    """Returns {kernel name: (milliseconds, launches)} accumulated since the last reset."""
    lib = _lib.load()
    out = {}
    i = 0
    while True:
        name, ms, n = ctypes.c_char_p(), ctypes.c_double(), ctypes.c_int64()
        if lib.gsa_profile_read(i, ctypes.byref(name), ctypes.byref(ms), ctypes.byref(n)) != 0:
            break
        out[name.value.decode()] = (ms.value, n.value)
        i += 1
    return out
