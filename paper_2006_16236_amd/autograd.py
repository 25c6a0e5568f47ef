"""torch.autograd front end of the C ABI: two differentiable functions.

Marshalling only: forward and backward are the library's kernels (la_causal_fwd / la_causal_bwd,
la_global_fwd / la_global_bwd); this file allocates the outputs and tells autograd what to keep.
What is kept for the backward is Q, K, V, the denominators [B, H, N] and the forward's workspace
(the running sums at the segment borders): the attention output itself is not needed, and no
per-position state is stored (the constant-memory backward of section 3.3.1).
"""
from __future__ import annotations

import torch

from . import binding as _b


class _CausalLinearAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, Q, K, V, eps, token_major):
        Q, K, V = Q.contiguous(), K.contiguous(), V.contiguous()
        O = torch.empty_like(V)
        if token_major:     # [B, N, H, .]
            B, N, H = Q.shape[:3]
            den = torch.empty((B, H, N), dtype=torch.float32, device=Q.device)
            ws = _b.la_causal_fwd_bnhd(Q, K, V, O, den, eps)
        else:
            den = torch.empty(Q.shape[:-1], dtype=torch.float32, device=Q.device)
            ws = _b.la_causal_fwd(Q, K, V, O, den, eps)
        ctx.save_for_backward(Q, K, V, den, ws)
        ctx.eps, ctx.token_major = eps, token_major
        return O

    @staticmethod
    def backward(ctx, dO):
        Q, K, V, den, ws = ctx.saved_tensors
        dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
        bwd = _b.la_causal_bwd_bnhd if ctx.token_major else _b.la_causal_bwd
        bwd(Q, K, V, None, den, dO.contiguous(), dQ, dK, dV, ctx.eps, fwd_ws=ws)
        return dQ, dK, dV, None, None


class _LinearAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, Q, K, V, eps, token_major):
        Q, K, V = Q.contiguous(), K.contiguous(), V.contiguous()
        O = torch.empty_like(V)
        if token_major:     # [B, N, H, .]
            B, N, H = Q.shape[:3]
            den = torch.empty((B, H, N), dtype=torch.float32, device=Q.device)
            ws = _b.la_global_fwd_bnhd(Q, K, V, O, eps, den=den)
        else:
            den = torch.empty(Q.shape[:-1], dtype=torch.float32, device=Q.device)
            ws = _b.la_global_fwd(Q, K, V, O, eps, den=den)
        ctx.save_for_backward(Q, K, V, den, ws)
        ctx.eps, ctx.token_major = eps, token_major
        return O

    @staticmethod
    def backward(ctx, dO):
        Q, K, V, den, ws = ctx.saved_tensors
        dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
        bwd = _b.la_global_bwd_bnhd if ctx.token_major else _b.la_global_bwd
        bwd(Q, K, V, None, den, dO.contiguous(), dQ, dK, dV, ctx.eps, fwd_ws=ws)
        return dQ, dK, dV, None, None


def causal_linear_attention(Q, K, V, eps: float = 1e-6, layout: str = "bhnd"):
    """Causal linear attention (eq. 9-12) of Q, K [B, H, N, D], V [B, H, N, M] with
    phi(x) = elu(x) + 1; differentiable with respect to Q, K, V.  layout="bnhd": the tensors
    (and the result) are [B, N, H, .], as a fused projection produces them; nothing is transposed."""
    if layout not in ("bhnd", "bnhd"):
        raise ValueError("layout must be 'bhnd' or 'bnhd'")
    return _CausalLinearAttention.apply(Q, K, V, float(eps), layout == "bnhd")


def linear_attention(Q, K, V, eps: float = 1e-6, layout: str = "bhnd"):
    """Non-causal linear attention (eq. 4-6); differentiable with respect to Q, K, V.
    layout as for causal_linear_attention."""
    if layout not in ("bhnd", "bnhd"):
        raise ValueError("layout must be 'bhnd' or 'bnhd'")
    return _LinearAttention.apply(Q, K, V, float(eps), layout == "bnhd")
