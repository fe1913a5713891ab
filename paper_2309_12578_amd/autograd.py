"""torch.autograd front end of the sparse attention (Section 4.3, "Integration of GPU kernels with
PyTorch": the shared library is loaded once and a custom autograd function calls its forward and
backward entry points).  Glue only: both directions run in libspion's kernels."""
from __future__ import annotations

import torch

from . import binding as _b


class _SpionAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, Q, K, V, pattern, scale, flags):
        Q, K, V = Q.contiguous(), K.contiguous(), V.contiguous()
        O, LSE = _b.attn_fwd(Q, K, V, pattern, scale=scale, flags=flags)
        ctx.save_for_backward(Q, K, V, O, LSE)
        ctx.pattern, ctx.scale, ctx.flags = pattern, scale, flags
        return O

    @staticmethod
    def backward(ctx, dO):
        Q, K, V, O, LSE = ctx.saved_tensors
        dQ, dK, dV = _b.attn_bwd(Q, K, V, O, dO.contiguous(), LSE, ctx.pattern, scale=ctx.scale,
                                 flags=ctx.flags)
        return dQ, dK, dV, None, None, None


def sparse_attention(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, pattern: _b.Pattern,
                     scale: float = 0.0, flags: int = 0) -> torch.Tensor:
    """Eq. 5 on the kept blocks of `pattern` for Q, K, V of shape [B, H, L, 64] (bf16 or fp32);
    differentiable with respect to Q, K and V."""
    return _SpionAttention.apply(Q, K, V, pattern, scale, flags)
