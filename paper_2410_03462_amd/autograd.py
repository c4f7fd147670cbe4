"""Differentiable wrapper: GRF-masked linear attention as a ``torch.autograd.Function``.

Plumbing only: forward and backward are the library's entry points (``grf_sample``,
``grf_masked_linear_attention_fused`` / ``grf_asymmetric_masked_attention`` and their backward
calls); this module decides what to save between them.  The modulation vector ``f`` of Alg. 1 is
a learnable tensor: its gradient comes from ``grf_sample_backward`` over the same walks.
"""
from __future__ import annotations

import torch

from . import binding as grf


class _GrfAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, Q, K, V, f, graph, p_halt, n_walks, seed, feature_map, asymmetric):
        f2 = f.detach().reshape(-1, f.shape[-1]).to("cpu", torch.float32).contiguous()
        phi = grf.grf_sample(graph, f2.numpy(), p_halt, n_walks, seed)
        if asymmetric:
            out, _, den = grf.grf_asymmetric_masked_attention(Q, K, V, phi, feature_map, return_num_den=True)
        else:
            out, _, den = grf.grf_masked_linear_attention_fused(Q, K, V, phi, feature_map, return_num_den=True)
        ctx.save_for_backward(Q, K, V, out, den)
        ctx.phi, ctx.graph = phi, graph
        ctx.walk = (int(f2.shape[1]), float(p_halt), int(n_walks), int(seed))
        ctx.feature_map, ctx.asymmetric, ctx.f_meta = feature_map, asymmetric, (f.shape, f.dtype, f.device)
        return out

    @staticmethod
    def backward(ctx, d_out):
        Q, K, V, out, den = ctx.saved_tensors
        call = grf.grf_asymmetric_masked_attention_backward if ctx.asymmetric else grf.grf_masked_linear_attention_backward
        dQ, dK, dV, dphi = call(Q, K, V, ctx.phi, out, den, d_out.contiguous().float(), ctx.feature_map,
                                want_dphi=ctx.needs_input_grad[3])
        df = None
        if ctx.needs_input_grad[3]:
            f_len, p_halt, n_walks, seed = ctx.walk
            shape, dtype, device = ctx.f_meta
            df = grf.grf_sample_backward(ctx.graph, f_len, p_halt, n_walks, seed, ctx.phi, dphi).reshape(shape).to(device, dtype)
        return dQ.to(Q.dtype), dK.to(K.dtype), dV.to(V.dtype), df, None, None, None, None, None, None


def grf_attention(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, f: torch.Tensor, graph: grf.DeviceGraph,
                  p_halt: float, n_walks: int, seed: int, feature_map: str = "relu", asymmetric: bool = False) -> torch.Tensor:
    """out [B,H,n,d] fp32, differentiable in Q, K, V and f.

    ``f`` is [f_len] (one modulation vector shared by the heads) or [H, f_len] (one per head, same walks).
    ``asymmetric`` selects the asymmetric-GRF estimator, where f holds the mask's own coefficients.
    The walks are a function of (graph, p_halt, n_walks, seed): keep the seed fixed for a frozen graph,
    change it to resample.
    """
    return _GrfAttention.apply(Q, K, V, f, graph, p_halt, n_walks, seed, feature_map, asymmetric)
