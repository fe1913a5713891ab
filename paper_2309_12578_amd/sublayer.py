"""The sparse multi-head-attention sub-layer of Algorithm 5 as a torch module.

Glue around the library: LayerNorm, the four projections (plain torch / hipBLASLt GEMMs), the head
split, dropout and the residual are torch ops; lines 4-7 of Algorithm 5 (SDDMM, sparse softmax, SpMM
for every head) are one call into libspion through `sparse_attention`, forward and backward.
"""
from __future__ import annotations

import torch
from torch import nn

from . import binding as _b
from .autograd import sparse_attention

HEAD_DIM = 64   # the only head dimension the kernels are built for


class SparseMHA(nn.Module):
    """O = dropout(concat_h(sparse_attention(Q_h, K_h, V_h, P)) W^O) + E with
    Q, K, V = LayerNorm(E) W^{Q,K,V} (Algorithm 5).  `embed_dim` must be 64 * heads."""

    def __init__(self, embed_dim: int, heads: int, dropout: float = 0.0, bias: bool = False,
                 device=None, dtype=None):
        super().__init__()
        if embed_dim != heads * HEAD_DIM:
            raise ValueError("embed_dim must be %d * heads" % HEAD_DIM)
        kw = dict(device=device, dtype=dtype)
        self.heads = heads
        self.norm = nn.LayerNorm(embed_dim, **kw)
        self.w_qkv = nn.Linear(embed_dim, 3 * embed_dim, bias=bias, **kw)   # W^Q | W^K | W^V
        self.w_o = nn.Linear(embed_dim, embed_dim, bias=bias, **kw)
        self.drop = nn.Dropout(dropout)

    def forward(self, E: torch.Tensor, pattern: _b.Pattern, flags: int = 0) -> torch.Tensor:
        """E: [B, L, embed_dim] on the GPU (bf16 or fp32); pattern: the layer's sparsity pattern."""
        B, L, D = E.shape
        X = self.norm(E)
        qkv = self.w_qkv(X).view(B, L, 3, self.heads, HEAD_DIM)
        # [B, H, L, 64] contiguous per tensor: the layout the kernels take
        Q, K, V = [qkv[:, :, i].transpose(1, 2).contiguous() for i in range(3)]
        S = sparse_attention(Q, K, V, pattern, flags=flags)               # lines 4-7, all heads at once
        S = S.transpose(1, 2).reshape(B, L, D)                            # concatenate the heads
        return self.drop(self.w_o(S)) + E
