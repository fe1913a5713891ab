"""Operation and byte counts used by the benchmark (no GPU code here).

Paper counts (Section 4.4, "Computational Complexity Analysis Comparison"): dense attention per
head needs 2 L^2 (2D+1) - L (D+1) operations, the sparse one 2 C (2D+1) - L (D+1) with C kept
score entries; SDDMM alone needs C (2D - 1).

Benchmark counts: a kept block is a dense bs x bs tile, each of the six useful tile products
(forward S = Q K^T and O = P V; backward dV, dP, dQ, dK) costs 2 bs^2 d FLOP.  Recomputing S in
the backward pass and the softmax exponentials are not counted as useful work.
"""
from __future__ import annotations

MI355X_HBM_GBPS = 8000.0          # published HBM3E peak, GB/s
MI355X_MFMA_TFLOPS = {"bf16": 2500.0, "f32": 157.3}   # published dense MFMA peaks


def paper_ops_dense(L: int, D: int) -> int:
    return 2 * L * L * (2 * D + 1) - L * (D + 1)


def paper_ops_sparse(L: int, D: int, C: int) -> int:
    return 2 * C * (2 * D + 1) - L * (D + 1)


def paper_ops_sddmm(D: int, C: int) -> int:
    return C * (2 * D - 1)


def useful_flops(nnzb: int, bs: int, d: int, bh: int, products: int = 6) -> int:
    """Useful FLOP of `products` tile products over all kept blocks of all heads.
    forward = 2 products, backward = 4, forward + backward = 6."""
    return 2 * bs * bs * d * nnzb * bh * products


def tensor_bytes(bh: int, L: int, d: int, elem_bytes: int) -> int:
    return bh * L * d * elem_bytes


def algorithmic_bytes(kernel: str, bh: int, L: int, d: int, elem_bytes: int) -> int:
    """Compulsory HBM traffic of one launch: every tensor the step needs, moved exactly once.

    fwd        reads Q, K, V; writes O and LSE
    bwd        reads Q, K, V, O, dO, LSE; writes dQ, dK, dV (the whole backward call)
    bwd_query  the query side of the backward run alone: reads Q, K, V, O, dO, LSE; writes dQ
    bwd_key    the key side run alone: reads Q, K, V, O, dO, LSE; writes dK, dV
    path       forward + backward of an ideal fused implementation: reads Q, K, V (fwd), writes O;
               reads Q, K, V, O, dO, writes dQ, dK, dV (12 tensor passes) plus LSE / delta vectors
    """
    t = tensor_bytes(bh, L, d, elem_bytes)
    vec = bh * L * 4
    if kernel == "fwd":
        return 4 * t + vec
    if kernel == "bwd":
        return 8 * t + vec
    if kernel == "bwd_query":
        return 6 * t + vec
    if kernel == "bwd_key":
        return 7 * t + vec
    if kernel == "path":
        return 12 * t + 2 * vec
    raise ValueError(kernel)
