"""torch.autograd front end over gsa_fwd / gsa_bwd (argument marshalling only: every step runs in libgsa).

    o = gsa_attention(q, k, v, g)                               # Eq. (gsa), chunkwise on the GPU
    o, (KT, VT) = gsa_attention(q, k, v, g, K0=K0, V0=V0, output_final_state=True)

Gradients flow to q, k, v, g, the optional write intensities s and the optional initial memories; gradients
arriving at the final memories are passed on to the backward call.  recompute=False keeps the forward's
per-chunk memories (the workspace, held by the autograd context until the backward has run) instead of
recomputing them in the backward: the kernel "without recomputation" of Section 4.1.4.
"""
import torch

from . import api


class _Gsa(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, k, v, g, s, K0, V0, scale, cu_seqlens, readout, gate_tau, feature_map, want_final, keep):
        ws = None
        if keep:
            ws = api.alloc_workspace(api.make_problem(q, v, g, scale, cu_seqlens, keep_states=True), True, q.device)
        o, z, KT, VT = api.gsa_fwd(q, k, v, g, K0=K0, V0=V0, scale=scale, cu_seqlens=cu_seqlens, save_z=True,
                                   final_state=want_final, s=s, readout=readout, gate_tau=gate_tau,
                                   feature_map=feature_map, workspace=ws, keep_states=keep)
        ctx.save_for_backward(q, k, v, g, z, s, K0, V0)
        ctx.opts = (scale, cu_seqlens, readout, gate_tau, feature_map)
        ctx.kept = ws   # not an autograd tensor: plain scratch that must survive, untouched, until backward
        if want_final:
            return o, KT, VT
        return o

    @staticmethod
    def backward(ctx, dO, dKT=None, dVT=None):
        q, k, v, g, z, s, K0, V0 = ctx.saved_tensors
        scale, cu_seqlens, readout, gate_tau, feature_map = ctx.opts
        need_init = (K0 is not None and ctx.needs_input_grad[5]) or (V0 is not None and ctx.needs_input_grad[6])
        res = api.gsa_bwd(q, k, v, g, z, dO.contiguous(), K0=K0, V0=V0,
                          dKT=None if dKT is None else dKT.contiguous(),
                          dVT=None if dVT is None else dVT.contiguous(), scale=scale, cu_seqlens=cu_seqlens,
                          initial_state_grad=need_init, s=s, readout=readout, gate_tau=gate_tau,
                          feature_map=feature_map, workspace=ctx.kept, keep_states=ctx.kept is not None)
        ctx.kept = None   # the backward has used the kept memories (and overwritten parts of the workspace)
        dq, dk, dv, dg, dK0, dV0 = res[:6]
        ds = res[6] if s is not None else None
        return (dq, dk, dv, dg, ds, dK0 if K0 is not None else None, dV0 if V0 is not None else None,
                None, None, None, None, None, None, None)


def gsa_attention(q, k, v, g, s=None, K0=None, V0=None, scale=1.0, cu_seqlens=None, readout="softmax", gate_tau=0.0,
                  feature_map="none", output_final_state=False, recompute=True):
    """q,k [B,T,H,d_k], v [B,T,H,d_v] (bf16 or fp32), g [B,T,H,m] fp32 log forget gates (or gate logits with
    gate_tau > 0); s optional write intensities [B,T,H,m]; K0,V0 optional initial memories [n,H,m,d] fp32;
    feature_map "swish": q, k, v are raw projections, x*sigmoid(x) is applied inside the kernels.
    recompute=False: the backward reads the forward's per-chunk memories instead of recomputing them (one
    backward pass per forward: the kept workspace is consumed).
    Returns o, or (o, (KT, VT)) with output_final_state."""
    out = _Gsa.apply(q.contiguous(), k.contiguous(), v.contiguous(), g.contiguous(),
                     None if s is None else s.contiguous(), K0, V0, float(scale), cu_seqlens, readout,
                     float(gate_tau), feature_map, bool(output_final_state), not recompute)
    if output_final_state:
        return out[0], (out[1], out[2])
    return out
