"""Pins for the attention half of the CPU oracle (no GPU needed).

The oracle's masked attention is checked against the dense definition (Eq. 1) written
independently in numpy, against torch's autograd on CPU (a library routine), against central
finite differences, and against invariants that any softmax attention obeys.
"""
import numpy as np
import pytest
import torch

import oracle


def _rand(bh, L, d, seed):
    rng = np.random.default_rng(seed)
    return [rng.standard_normal((bh, L, d)) for _ in range(4)]


def _mask(L, bs, density, seed):
    rng = np.random.default_rng(seed)
    nb = L // bs
    m = (rng.random((nb, nb)) < density).astype(np.uint8)
    m[np.arange(nb), np.arange(nb)] = 1
    return np.kron(m, np.ones((bs, bs), dtype=np.uint8))


def dense_attention_numpy(Q, K, V, scale):
    S = scale * np.einsum("bid,bjd->bij", Q, K)
    S = S - S.max(axis=-1, keepdims=True)
    E = np.exp(S)
    A = E / E.sum(axis=-1, keepdims=True)
    return np.einsum("bij,bjd->bid", A, V)


def test_all_ones_mask_reproduces_dense_attention():
    Q, K, V, _ = _rand(3, 40, 16, 0)
    P = np.ones((40, 40), dtype=np.uint8)
    O, LSE = oracle.attn_fwd(Q, K, V, P)
    ref = dense_attention_numpy(Q, K, V, 0.25)
    assert np.allclose(O, ref, rtol=1e-12, atol=1e-13)
    S = 0.25 * np.einsum("bid,bjd->bij", Q, K)
    assert np.allclose(LSE, np.log(np.exp(S).sum(-1)), rtol=1e-12)


def test_default_scale_is_inverse_sqrt_head_dim_and_scale_is_used():
    Q, K, V, _ = _rand(1, 8, 64, 1)
    P = np.ones((8, 8), dtype=np.uint8)
    O, _ = oracle.attn_fwd(Q, K, V, P)
    assert np.allclose(O, dense_attention_numpy(Q, K, V, 0.125), rtol=1e-12)
    O2, _ = oracle.attn_fwd(Q, K, V, P, scale=0.5)
    assert np.allclose(O2, dense_attention_numpy(Q, K, V, 0.5), rtol=1e-12)


def test_kept_probabilities_sum_to_one_and_masked_are_zero():
    Q, K, V, _ = _rand(2, 32, 8, 2)
    P = _mask(32, 4, 0.3, 2)
    for bh in range(2):
        for i in (0, 5, 31):
            p = oracle.attn_probs_row(Q, K, P, bh, i)
            assert abs(p.sum() - 1.0) < 1e-12
            assert np.all(p[P[i] == 0] == 0.0)
            assert np.all(p[P[i] == 1] > 0.0)


def test_masked_keys_and_values_do_not_contribute():
    Q, K, V, _ = _rand(1, 32, 8, 3)
    P = _mask(32, 8, 0.3, 3)
    O, _ = oracle.attn_fwd(Q, K, V, P)
    i = 9
    K2, V2 = K.copy(), V.copy()
    dead = np.where(P[i] == 0)[0]
    assert dead.size > 0
    K2[0, dead] += 100.0
    V2[0, dead] -= 55.0
    O2, _ = oracle.attn_fwd(Q, K2, V2, P)
    assert np.array_equal(O[0, i], O2[0, i])


def test_block_diagonal_mask_is_independent_small_attentions():
    L, bs, d = 24, 6, 8
    Q, K, V, _ = _rand(2, L, d, 4)
    P = np.kron(np.eye(L // bs, dtype=np.uint8), np.ones((bs, bs), dtype=np.uint8))
    O, _ = oracle.attn_fwd(Q, K, V, P)
    for g in range(L // bs):
        s = slice(g * bs, (g + 1) * bs)
        ref = dense_attention_numpy(Q[:, s], K[:, s], V[:, s], 1 / np.sqrt(d))
        assert np.allclose(O[:, s], ref, rtol=1e-12, atol=1e-13)


def _torch_masked_attention(Q, K, V, P, scale):
    q, k, v = [torch.tensor(t, dtype=torch.float64, requires_grad=True) for t in (Q, K, V)]
    s = scale * q @ k.transpose(-1, -2)
    s = s.masked_fill(torch.tensor(P == 0), float("-inf"))
    o = torch.softmax(s, dim=-1) @ v
    return q, k, v, o


@pytest.mark.parametrize("density", [1.0, 0.35])
def test_forward_and_gradients_match_torch_autograd(density):
    L, bs, d = 48, 8, 16
    Q, K, V, dO = _rand(2, L, d, 5)
    P = _mask(L, bs, density, 5)
    scale = 1 / np.sqrt(d)
    q, k, v, o = _torch_masked_attention(Q, K, V, P, scale)
    o.backward(torch.tensor(dO))
    O, _ = oracle.attn_fwd(Q, K, V, P)
    dQ, dK, dV = oracle.attn_bwd(Q, K, V, dO, P)
    assert np.allclose(O, o.detach().numpy(), rtol=1e-11, atol=1e-12)
    assert np.allclose(dQ, q.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(dK, k.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(dV, v.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_gradients_match_central_finite_differences():
    L, bs, d, h = 32, 8, 8, 1e-5
    Q, K, V, dO = _rand(1, L, d, 6)
    P = _mask(L, bs, 0.4, 6)
    dQ, dK, dV = oracle.attn_bwd(Q, K, V, dO, P)

    def loss(q, k, v):
        o, _ = oracle.attn_fwd(q, k, v, P)
        return float((o * dO).sum())

    rng = np.random.default_rng(60)
    for name, X, G in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV)):
        for _ in range(12):
            idx = (0, int(rng.integers(L)), int(rng.integers(d)))
            Xp, Xm = X.copy(), X.copy()
            Xp[idx] += h
            Xm[idx] -= h
            args_p = {"Q": (Xp, K, V), "K": (Q, Xp, V), "V": (Q, K, Xp)}[name]
            args_m = {"Q": (Xm, K, V), "K": (Q, Xm, V), "V": (Q, K, Xm)}[name]
            fd = (loss(*args_p) - loss(*args_m)) / (2 * h)
            assert fd == pytest.approx(G[idx], rel=1e-6, abs=1e-8), (name, idx)


def test_key_gradients_sum_to_zero_over_each_rows_kept_set():
    # adding one vector to every key shifts each score row by a constant, which softmax ignores:
    # hence sum_j dS_ij = 0 and, with an all-ones mask, sum_j dK_j = 0.
    Q, K, V, dO = _rand(2, 24, 8, 7)
    P = np.ones((24, 24), dtype=np.uint8)
    _, dK, _ = oracle.attn_bwd(Q, K, V, dO, P)
    assert np.allclose(dK.sum(axis=1), 0.0, atol=1e-12)


def test_paper_denominator_flag():
    # Algorithm 6 adds exp(-max) * (L - kept) to the row sum: masked entries count as score 0.
    L, bs, d = 32, 8, 8
    Q, K, V, dO = _rand(2, L, d, 8)
    scale = 1 / np.sqrt(d)
    ones = np.ones((L, L), dtype=np.uint8)
    a, _ = oracle.attn_fwd(Q, K, V, ones)
    b, _ = oracle.attn_fwd(Q, K, V, ones, flags=oracle.ATTN_PAPER_DENOM)
    assert np.array_equal(a, b)                       # identical for an all-ones pattern
    P = _mask(L, bs, 0.4, 8)
    S = scale * np.einsum("bid,bjd->bij", Q, K) * P   # literal Eq. 5: (P>0) .* QK^T, then softmax
    E = np.exp(S - S.max(-1, keepdims=True))
    A = E / E.sum(-1, keepdims=True) * P              # only kept entries are stored
    ref = np.einsum("bij,bjd->bid", A, V)
    O, LSE = oracle.attn_fwd(Q, K, V, P, flags=oracle.ATTN_PAPER_DENOM)
    assert np.allclose(O, ref, rtol=1e-11, atol=1e-13)
    # the row statistic of that variant: log of the literal Eq. 5 row sum (masked entries are exp(0))
    assert np.allclose(LSE, np.log(np.exp(S).sum(-1)), rtol=1e-12, atol=0)
    kept = P.sum(-1)                                   # and, term by term, Algorithm 6's sum
    ref_sum = (np.exp(scale * np.einsum("bid,bjd->bij", Q, K)) * P).sum(-1) + (L - kept)[None, :]
    assert np.allclose(np.exp(LSE), ref_sum, rtol=1e-12, atol=0)
    # a row that keeps nothing still has the L masked entries in its denominator
    P0 = P.copy()
    P0[8:16, :] = 0
    O0, LSE0 = oracle.attn_fwd(Q, K, V, P0, flags=oracle.ATTN_PAPER_DENOM)
    assert np.all(O0[:, 8:16] == 0.0)
    # gradient of that variant against torch autograd of the same expression
    q, k, v = [torch.tensor(t, requires_grad=True) for t in (Q, K, V)]
    Pt = torch.tensor(P, dtype=torch.float64)
    o = (torch.softmax(scale * (q @ k.transpose(-1, -2)) * Pt, dim=-1) * Pt) @ v
    o.backward(torch.tensor(dO))
    dQ, dK, dV = oracle.attn_bwd(Q, K, V, dO, P, flags=oracle.ATTN_PAPER_DENOM)
    assert np.allclose(dQ, q.grad.numpy(), rtol=1e-9, atol=1e-12)
    assert np.allclose(dK, k.grad.numpy(), rtol=1e-9, atol=1e-12)
    assert np.allclose(dV, v.grad.numpy(), rtol=1e-9, atol=1e-12)


def test_empty_row_gives_zero_output():
    Q, K, V, dO = _rand(1, 8, 4, 9)
    P = np.ones((8, 8), dtype=np.uint8)
    P[3, :] = 0
    O, LSE = oracle.attn_fwd(Q, K, V, P)
    assert np.all(O[0, 3] == 0.0) and LSE[0, 3] == -np.inf
    dQ, dK, dV = oracle.attn_bwd(Q, K, V, dO, P)
    assert np.all(dQ[0, 3] == 0.0) and np.all(np.isfinite(dK)) and np.all(np.isfinite(dV))
