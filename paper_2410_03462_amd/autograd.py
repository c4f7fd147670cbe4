"""Differentiable wrapper: GRF-masked linear attention as a ``torch.autograd.Function``.

Plumbing only: forward and backward are the library's entry points (``grf_sample``,
``grf_masked_linear_attention_fused`` / ``grf_asymmetric_masked_attention`` and their backward
calls); this module decides what to save between them.  The modulation vector ``f`` of Alg. 1 is
a learnable tensor: its gradient comes from ``grf_sample_backward`` over the same walks.
"""
from __future__ import annotations

import numpy as np
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


class _FrozenWalkAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, Q, K, V, f, state):
        phi, prepared = state._refresh(f)
        fm = state.feature_map
        if state.asymmetric:
            out, _, den = grf.grf_asymmetric_masked_attention(Q, K, V, phi, fm, return_num_den=True)
        else:
            out, _, den = grf.grf_masked_linear_attention_fused(Q, K, V, phi, fm, prepared=prepared, return_num_den=True)
        ctx.save_for_backward(Q, K, V, out, den)
        ctx.state, ctx.f_meta = state, (f.shape, f.dtype)
        return out

    @staticmethod
    def backward(ctx, d_out):
        Q, K, V, out, den = ctx.saved_tensors
        st = ctx.state
        d_out = d_out.contiguous().float()
        if st.asymmetric:
            dQ, dK, dV, dphi = grf.grf_asymmetric_masked_attention_backward(Q, K, V, st.phi, out, den, d_out, st.feature_map,
                                                                            want_dphi=ctx.needs_input_grad[3])
        else:
            dQ, dK, dV, dphi = grf.grf_masked_linear_attention_backward(Q, K, V, st.phi, out, den, d_out, st.feature_map,
                                                                        want_dphi=ctx.needs_input_grad[3], prepared=st.prepared)
        df = None
        if ctx.needs_input_grad[3]:
            shape, dtype = ctx.f_meta
            df = grf.grf_sample_backward(st.graph, st.f_len, st.p_halt, st.n_walks, st.seed, st.phi, dphi).reshape(shape).to(dtype)
        return dQ.to(Q.dtype), dK.to(K.dtype), dV.to(V.dtype), df, None


class FrozenWalkAttention:
    """GRF-masked attention over frozen walks (Sec. 4: the walks of a graph are sampled once per head and layer, the
    modulation f stays learnable).  Plumbing only, as above; what it keeps between calls is what does not depend on f:
    the pattern of Phi_hat, its column lists (``grf_phi_prepare``) and the sampler's workspace.  A call refreshes the
    values of Phi_hat from the current f on the device (``grf_sample_async``: the same walks from the counter-based
    stream, no host synchronisation), takes them over into the lists (``grf_phi_prepare_values``) and runs the prepared
    forms of the attention calls; results are the bits that ``grf_attention`` returns for the same arguments.

    ``f`` passed to a call is a CUDA fp32 tensor [f_len] or [H, f_len] with ``n_f`` rows in all.  Calls on one instance
    share its buffers: finish the backward pass of a call before the next forward pass with another f.
    """

    def __init__(self, graph: grf.DeviceGraph, f_len: int, n_f: int, p_halt: float, n_walks: int, seed: int,
                 feature_map: str = "relu", asymmetric: bool = False):
        self.graph, self.f_len, self.n_f = graph, int(f_len), int(n_f)
        self.p_halt, self.n_walks, self.seed = float(p_halt), int(n_walks), int(seed)
        self.feature_map, self.asymmetric = feature_map, bool(asymmetric)
        L = grf.lib()
        dev = graph.row_ptr.device
        bound = int(L.grf_sample_nnz_bound(graph.n, self.n_walks, self.f_len))
        self.phi = grf.Phi.empty(graph.n, bound, self.n_f, dev)
        self.sample_ws = torch.empty(max(int(L.grf_sample_workspace_bytes(graph.n, self.n_walks, self.f_len, self.n_f)), 1),
                                     dtype=torch.uint8, device=dev)
        # the pattern does not depend on f: one synchronising call with any f tells the number of entries
        probe = grf.grf_sample(graph, np.ones((self.n_f, self.f_len), np.float32), self.p_halt, self.n_walks, self.seed,
                               out=self.phi, workspace=self.sample_ws)
        self.nnz = int(probe.nnz)
        self.prepared = None

    def _refresh(self, f: torch.Tensor):
        f2 = f.detach().reshape(-1, f.shape[-1]).to(torch.float32).contiguous()
        if tuple(f2.shape) != (self.n_f, self.f_len) or not f2.is_cuda:
            raise ValueError(f"f must be a CUDA tensor of {self.n_f} x {self.f_len} values")
        grf.grf_sample_async(self.graph, f2, self.p_halt, self.n_walks, self.seed, out=self.phi, workspace=self.sample_ws)
        self.phi.nnz = self.nnz          # the async call reports its capacity bound; the pattern's size is known
        if not self.asymmetric:
            if self.prepared is None:
                self.prepared = grf.grf_phi_prepare(self.phi)
            else:
                grf.grf_phi_prepare_values(self.phi, self.prepared)
        return self.phi, self.prepared

    def __call__(self, Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, f: torch.Tensor) -> torch.Tensor:
        return _FrozenWalkAttention.apply(Q, K, V, f, self)
