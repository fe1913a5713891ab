"""GPU parity: libspion (through its C ABI) against the CPU oracle on the same seeded inputs.

Bars: pattern outputs (pool_sum, fl_out, BSR, BSC, nnzb) bit-exact; attention outputs and
gradients within 1e-5 (fp32) / 2e-2 (bf16), both as relative Frobenius error and as
max|x - ref| / max|ref|, against the fp64 oracle fed the same (already rounded) input values.
"""
import functools

import numpy as np
import pytest
import torch

import oracle
import spion_inputs as si

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}


@pytest.fixture(scope="module")
def sp():
    import paper_2309_12578_amd as sp
    sp.load()
    return sp


def _dev(x, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    return t if dtype is None else t.to(dtype)


def _torch_dtype(name):
    return torch.float32 if name == "f32" else torch.bfloat16


def _rel_errors(x, ref):
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    fro = np.linalg.norm(x - ref) / max(np.linalg.norm(ref), 1e-300)
    mx = np.abs(x - ref).max() / max(np.abs(ref).max(), 1e-300)
    return fro, mx


@functools.lru_cache(maxsize=2)
def _workload_inputs(name):
    """Q, K, V, dO and the score map averaged over ALL (batch, head) slices: the very map, and so
    the very index, that the benchmark times."""
    w = si.workload(name)
    Q, K, V, dO = si.make_qkv_do(w)
    return Q, K, V, dO, si.make_score_map(w, Q, K)


def _check_pattern(sp, A, block, filt, mode, value, flags=0, variant="CF"):
    ref = oracle.generate_pattern(A, block, filt, mode, value, variant=variant)
    pat = sp.generate_pattern(_dev(A), block, filt, mode, value, flags=flags)
    torch.cuda.synchronize()
    n = ref["nnzb"]
    assert np.array_equal(pat.pool_sum.cpu().numpy(), ref["pool_sum"]), "pool_sum"
    assert np.array_equal(pat.fl_out.cpu().numpy(), ref["fl_out"]), "fl_out"
    assert pat.nnzb == n
    assert np.array_equal(pat.row_ptr.cpu().numpy(), ref["row_ptr"])
    assert np.array_equal(pat.col_idx.cpu().numpy()[:n], ref["col_idx"])
    assert np.array_equal(pat.col_ptr.cpu().numpy(), ref["col_ptr"])
    assert np.array_equal(pat.row_idx.cpu().numpy()[:n], ref["row_idx"])
    assert np.array_equal(pat.bsr_pos.cpu().numpy()[:n], ref["bsr_pos"])
    return pat, ref


# ------------------------------------------------------------------------------------------------
# pattern
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("name", [w.name for w in si.WORKLOADS])
def test_pattern_bit_exact_on_workloads(sp, name):
    w = si.workload(name)
    A = _workload_inputs(name)[4]
    pat, ref = _check_pattern(sp, A, w.block, w.filt, w.thresh_mode, w.thresh_value)
    dens = ref["nnzb"] / float(w.nb * w.nb)
    print(f"{name}: nnzb={ref['nnzb']} density={dens:.4f}")
    assert ref["nnzb"] == si.EXPECTED_NNZB[name]
    # the sparser variant (q = 1 - target density) of the same map
    w1 = si.workload(name, variant="one_minus_target")
    if w1.thresh_value != w.thresh_value:
        _check_pattern(sp, A, w.block, w.filt, w1.thresh_mode, w1.thresh_value)


@pytest.mark.parametrize("L,block,filt", [(64, 16, 1), (128, 16, 5), (256, 32, 31), (256, 64, 31),
                                          (512, 32, 63), (2048, 16, 9), (192, 64, 127)])
@pytest.mark.parametrize("mode,value", [(si.T_QUANTILE, 0.0), (si.T_QUANTILE, 0.7), (si.T_QUANTILE, 1.0),
                                        (si.T_MEAN_KSTD, 0.5), (si.T_ABS, 0.02)])
def test_pattern_bit_exact_on_random_maps_with_ties(sp, L, block, filt, mode, value):
    rng = np.random.default_rng(L * 7 + block + filt)
    # coarse values (multiples of 1/8 up to 1) make equal pooled sums and plateaus common
    A = (rng.integers(0, 9, size=(L, L)) / 8.0).astype(np.float32)
    A[rng.random((L, L)) < 0.5] = 0.0
    if mode == si.T_ABS:
        value = float(A.mean()) * filt * 1.1
    _check_pattern(sp, A, block, filt, mode, value)


def test_pattern_large_block_grid_uses_the_workspace_path(sp):
    # nb = 256: the cell arrays no longer fit in LDS and live in the caller's workspace
    L, block = 4096, 16
    rng = np.random.default_rng(17)
    A = (rng.random((L, L), dtype=np.float32) ** 8).astype(np.float32)
    A[:, 1000:1016] += 0.5
    A = np.minimum(A, 1.0).astype(np.float32)
    _check_pattern(sp, A, block, 3, si.T_QUANTILE, 0.97)
    _check_pattern(sp, A, block, 1, si.T_MEAN_KSTD, 2.0)


def test_pattern_at_the_largest_block_grid(sp):
    # nb = 1024, the largest grid the library accepts: 2047 fill levels, one thread per block row
    L, block = 16384, 16
    rng = np.random.default_rng(5)
    A = rng.random((L, L), dtype=np.float32)
    for _ in range(3):
        np.multiply(A, A, out=A)                  # x^8: a few large scores on a faint background
    A[:, 5000:5016] += 0.5
    i = np.arange(L)
    A[i, i] += 0.4
    np.minimum(A, 1.0, out=A)
    _check_pattern(sp, A, block, 3, si.T_QUANTILE, 0.995)


def test_pattern_plateau_map_and_tiny_values(sp):
    L, block = 128, 16
    A = np.zeros((L, L), dtype=np.float32)        # every pooled value equal: all ties
    _check_pattern(sp, A, block, 1, si.T_ABS, -1.0)     # everything reachable is above t
    A[:] = 2.0 ** -41                               # rounds to 0 in fixed point (tie to even)
    A[5, 7] = 3 * 2.0 ** -41                        # rounds to 2
    A[9, 9] = -0.37
    _check_pattern(sp, A, block, 3, si.T_QUANTILE, 0.5)


@pytest.mark.parametrize("L,block,filt", [(256, 16, 7), (1024, 32, 31), (4096, 64, 31), (1024, 64, 127)])
def test_pattern_signed_scores(sp, L, block, filt):
    """Scores of both signs (the interface allows |a| <= 1): negative fixed-point values in the
    convolution, pooled sums on both sides of zero in the order statistic and in the fp64 threshold."""
    rng = np.random.default_rng(L + block)
    A = rng.uniform(-1.0, 1.0, size=(L, L)).astype(np.float32)
    A[rng.random((L, L)) < 0.3] *= 2.0 ** -20           # values that need the low fixed-point bits
    i = np.arange(L)
    A[i, (i * 7) % L] = -1.0
    A[(i * 5) % L, i] = 1.0
    _check_pattern(sp, A, block, filt, si.T_QUANTILE, 0.6)
    _check_pattern(sp, A, block, filt, si.T_MEAN_KSTD, 0.25)
    _check_pattern(sp, A, block, filt, si.T_ABS, -0.001)


def test_pattern_variants_no_fill_and_no_conv(sp):
    w = si.workload(1)
    Q, K, _, _ = si.make_qkv_do(w)
    A = si.make_score_map(w, Q, K)
    _check_pattern(sp, A, w.block, w.filt, si.T_QUANTILE, 0.9, flags=sp.SPION_PATTERN_NO_FILL, variant="C")
    _check_pattern(sp, A, w.block, 1, si.T_QUANTILE, 0.9, variant="F")


def test_pattern_halves_pool_only_then_from_pool(sp):
    """Eq. 3 + Eq. 4 alone (SPION_PATTERN_POOL_ONLY) and the rest of Algorithm 3 from a given pool_sum
    (SPION_PATTERN_FROM_POOL).  Conv and pool are linear and the sums exact integers, so the pool_sum
    maps of two halves of a batch add up to the map of the whole: the way the pattern would be made
    when the score maps are spread over several GPUs."""
    w = si.workload(2)
    Q, K, _, _ = si.make_qkv_do(w, bh_limit=8)
    A1 = si.make_score_map(w, Q[:4], K[:4]) * np.float32(0.5)
    A2 = si.make_score_map(w, Q[4:], K[4:]) * np.float32(0.5)
    nb = w.nb
    ref1 = oracle.pool_sum(oracle.conv_diag(oracle.quantize(A1), w.filt), w.block)
    ref2 = oracle.pool_sum(oracle.conv_diag(oracle.quantize(A2), w.filt), w.block)
    pools = []
    for A in (A1, A2):
        ps = torch.full((nb, nb), -1, dtype=torch.int64, device="cuda")
        ws = torch.empty(sp.spion_pattern_workspace_bytes(w.L, w.block), dtype=torch.uint8, device="cuda")
        sp.spion_pattern(_dev(A), w.L, w.block, w.filt, w.thresh_mode, w.thresh_value, None, None, None, None,
                         None, None, None, ps, ws, flags=sp.SPION_PATTERN_POOL_ONLY)
        pools.append(ps)
    assert np.array_equal(pools[0].cpu().numpy(), ref1) and np.array_equal(pools[1].cpu().numpy(), ref2)
    total = pools[0] + pools[1]
    t = oracle.threshold(ref1 + ref2, w.block, w.thresh_mode, w.thresh_value)
    ref = oracle.compact(oracle.fill(ref1 + ref2, t))
    i32 = dict(dtype=torch.int32, device="cuda")
    fl = torch.empty((nb, nb), dtype=torch.uint8, device="cuda")
    row_ptr, col_idx, nnzb = torch.empty(nb + 1, **i32), torch.empty(nb * nb, **i32), torch.empty(1, **i32)
    ws = torch.empty(sp.spion_pattern_workspace_bytes(w.L, w.block), dtype=torch.uint8, device="cuda")
    keep = total.clone()
    sp.spion_pattern(None, w.L, w.block, w.filt, w.thresh_mode, w.thresh_value, fl, row_ptr, col_idx, None, None,
                     None, nnzb, total, ws, flags=sp.SPION_PATTERN_FROM_POOL)
    n = int(nnzb.item())
    assert n == ref["nnzb"] and torch.equal(total, keep)                      # pool_sum is read only
    assert np.array_equal(row_ptr.cpu().numpy(), ref["row_ptr"])
    assert np.array_equal(col_idx.cpu().numpy()[:n], ref["col_idx"])
    assert np.array_equal(fl.cpu().numpy(), oracle.fill(ref1 + ref2, t))
    with pytest.raises(sp.SpionError) as e:                                    # the two flags exclude each other
        sp.spion_pattern(_dev(A1), w.L, w.block, w.filt, w.thresh_mode, w.thresh_value, fl, row_ptr, col_idx,
                         None, None, None, nnzb, total, ws,
                         flags=sp.SPION_PATTERN_FROM_POOL | sp.SPION_PATTERN_POOL_ONLY)
    assert e.value.code == -5


def test_copy_yardstick_moves_every_byte_once(sp):
    n = 3 * 16384 * 7
    src = torch.randint(0, 256, (n,), dtype=torch.uint8, device="cuda")
    dst = torch.zeros_like(src)
    sp.spion_copy_yardstick(src, dst, n)
    assert torch.equal(src, dst)
    with pytest.raises(sp.SpionError) as e:
        sp.spion_copy_yardstick(src, dst, n - 1)                               # not a multiple of 16 KB
    assert e.value.code == -2


def test_pattern_is_deterministic_across_runs(sp):
    w = si.workload(2)
    Q, K, _, _ = si.make_qkv_do(w, bh_limit=4)
    A = _dev(si.make_score_map(w, Q, K))
    first = sp.generate_pattern(A, w.block, w.filt, w.thresh_mode, w.thresh_value)
    for _ in range(5):
        again = sp.generate_pattern(A, w.block, w.filt, w.thresh_mode, w.thresh_value)
        assert torch.equal(first.fl_out, again.fl_out) and torch.equal(first.pool_sum, again.pool_sum)
        assert torch.equal(first.col_idx[:first.nnzb], again.col_idx[:again.nnzb])


# ------------------------------------------------------------------------------------------------
# producers of the pattern input
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n_maps,L", [(1, 64), (7, 264), (16, 1024)])
def test_score_mean_matches_oracle(sp, dtype, n_maps, L):
    rng = np.random.default_rng(n_maps * 1000 + L)
    maps = si.round_to_dtype(rng.random((n_maps, L, L), dtype=np.float32) ** 4, dtype)
    got = sp.score_mean(_dev(maps, _torch_dtype(dtype))).cpu().numpy().astype(np.float64)
    ref = oracle.score_mean(maps)
    # fp32 sequential sum of n_maps terms, then one division
    assert np.all(np.abs(got - ref) <= 1e-6 * np.abs(ref) + 1e-12), np.abs(got - ref).max()


@pytest.mark.parametrize("n", [16, 1000, 4099, 1024 * 1024, 4096 * 4096])
def test_frobenius_distance_matches_oracle(sp, n):
    rng = np.random.default_rng(n)
    a = rng.random(n, dtype=np.float32)
    b = (rng.random(n, dtype=np.float32) * 1.01).astype(np.float32)
    out = sp.frobenius_distance(_dev(a), _dev(b)).cpu().numpy()
    d, na, nb_ = oracle.frobenius_distance(a, b)
    assert out[1] == pytest.approx(na, rel=1e-12) and out[2] == pytest.approx(nb_, rel=1e-12)
    assert out[0] == pytest.approx(d, rel=1e-9, abs=1e-12 * na)
    again = sp.frobenius_distance(_dev(a), _dev(b)).cpu().numpy()
    assert np.array_equal(out, again)                     # fixed summation order


def test_pattern_from_gpu_averaged_map(sp):
    # the whole producer + pattern chain on device: per-head maps -> mean -> spion_pattern
    w = si.workload(1)
    rng = np.random.default_rng(5)
    heads = []
    Q, K, _, _ = si.make_qkv_do(w)
    base = si.make_score_map(w, Q, K)
    for h in range(6):
        heads.append((base * (0.5 + rng.random(base.shape, dtype=np.float32))).astype(np.float32))
    maps = np.minimum(np.stack(heads), 1.0).astype(np.float32)
    A_dev = sp.score_mean(_dev(maps))
    A = A_dev.cpu().numpy()
    pat = sp.generate_pattern(A_dev, w.block, w.filt, w.thresh_mode, w.thresh_value)
    ref = oracle.generate_pattern(A, w.block, w.filt, w.thresh_mode, w.thresh_value)
    assert np.array_equal(pat.fl_out.cpu().numpy(), ref["fl_out"])


# ------------------------------------------------------------------------------------------------
# attention
# ------------------------------------------------------------------------------------------------
def _pattern_from_mask(sp, fl, block):
    """Build the device index for a given block mask from the oracle's compaction (index bits are
    themselves checked against spion_pattern in the tests above)."""
    c = oracle.compact(fl)
    nb = fl.shape[0]
    pad = np.zeros(nb * nb, dtype=np.int32)

    def full(a):
        out = pad.copy()
        out[:a.size] = a
        return out

    return sp.Pattern(nb * block, block, _dev(fl), _dev(c["row_ptr"]), _dev(full(c["col_idx"])),
                      _dev(c["col_ptr"]), _dev(full(c["row_idx"])), _dev(full(c["bsr_pos"])),
                      _dev(np.array([c["nnzb"]], dtype=np.int32)),
                      torch.zeros((nb, nb), dtype=torch.int64, device="cuda"), c["nnzb"])


def _run_attention_case(sp, Q, K, V, dO, fl, block, dtype, flags=0, heads=None, scale=0.0):
    """Q.. are fp32 numpy [BH, L, d] holding values exactly representable in dtype."""
    BH, L, d = Q.shape
    tdt = _torch_dtype(dtype)
    pat = _pattern_from_mask(sp, fl, block)
    q, k, v, do = [_dev(t, tdt).view(1, BH, L, d) for t in (Q, K, V, dO)]
    O, LSE = sp.attn_fwd(q, k, v, pat, scale=scale, flags=flags)
    dQ, dK, dV = sp.attn_bwd(q, k, v, O, do, LSE, pat, scale=scale, flags=flags)
    torch.cuda.synchronize()
    sel = list(range(BH)) if heads is None else heads
    P = oracle.upsample(fl, block)
    sc = None if scale == 0.0 else scale
    oflags = oracle.ATTN_PAPER_DENOM if flags & sp.SPION_ATTN_PAPER_DENOM else 0
    rO, rLSE = oracle.attn_fwd(Q[sel], K[sel], V[sel], P, scale=sc, flags=oflags)
    rdQ, rdK, rdV = oracle.attn_bwd(Q[sel], K[sel], V[sel], dO[sel], P, scale=sc, flags=oflags)
    tol = TOL[dtype]
    got = {"O": O, "dQ": dQ, "dK": dK, "dV": dV}
    ref = {"O": rO, "dQ": rdQ, "dK": rdK, "dV": rdV}
    errs = {}
    for name in got:
        x = got[name].float().cpu().numpy().reshape(BH, L, d)[sel]
        assert np.all(np.isfinite(x)), name
        errs[name] = _rel_errors(x, ref[name])
    lse = LSE.cpu().numpy().reshape(BH, L)[sel]
    fin = np.isfinite(rLSE)
    assert np.array_equal(np.isneginf(lse), np.isneginf(rLSE))
    errs["LSE"] = ((np.abs(lse[fin] - rLSE[fin]).max() / max(np.abs(rLSE[fin]).max(), 1.0),) * 2
                   if fin.any() else (0.0, 0.0))          # a pattern may keep no block at all
    for name, (fro, mx) in errs.items():
        assert fro <= tol and mx <= tol, (name, fro, mx, tol)
    return errs


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("block", [16, 32, 64])
@pytest.mark.parametrize("density", [1.0, 0.3])
def test_attention_small_all_kernels(sp, dtype, block, density):
    nb, BH, d = 5, 3, 64          # several tiles per row plus ragged row/column lengths
    L = nb * block
    rng = np.random.default_rng(block * 10 + int(density * 10))
    Q, K, V, dO = [si.round_to_dtype(rng.standard_normal((BH, L, d), dtype=np.float32), dtype)
                   for _ in range(4)]
    fl = si.random_block_mask(nb, density, seed=block)
    errs = _run_attention_case(sp, Q, K, V, dO, fl, block, dtype)
    print(dtype, block, density, {k: f"{v[0]:.2e}" for k, v in errs.items()})


@pytest.mark.parametrize("block", [32, 64])
def test_attention_more_than_64_block_columns(sp, block):
    """96 block columns: the work-item lookup of the backward scans the column counts in two groups
    of 64; split columns (more than 16 kept rows) sit in both groups, next to short and empty-but-for-
    the-diagonal ones; 8 heads, so the workgroup-to-XCD mapping by head is in play."""
    nb, BH, d = 96, 8, 64
    L = nb * block
    rng = np.random.default_rng(block + 96)
    Q, K, V, dO = [si.round_to_dtype(rng.standard_normal((BH, L, d), dtype=np.float32), "bf16")
                   for _ in range(4)]
    fl = si.random_block_mask(nb, 0.06, seed=block + 5)
    fl[:, 7] = 1                                  # tall columns in the first group ...
    fl[rng.choice(nb, 40, replace=False), 33] = 1
    fl[:, 80] = 1                                 # ... and in the second
    fl[rng.choice(nb, 21, replace=False), 95] = 1
    fl[:, 70] = 0
    fl[70, 70] = 1                                # a column of one block
    _run_attention_case(sp, Q, K, V, dO, fl, block, "bf16", heads=[0, 5, 7])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_attention_degenerate_patterns(sp, dtype):
    block, nb, BH, d = 32, 4, 2, 64
    L = nb * block
    rng = np.random.default_rng(3)
    Q, K, V, dO = [si.round_to_dtype(rng.standard_normal((BH, L, d), dtype=np.float32), dtype)
                   for _ in range(4)]
    diag = np.eye(nb, dtype=np.uint8)                       # one block per row and column
    _run_attention_case(sp, Q, K, V, dO, diag, block, dtype)
    stripe = np.eye(nb, dtype=np.uint8)
    stripe[:, 2] = 1                                         # one full column: longest column walk
    stripe[1, :] = 1                                         # one full row
    _run_attention_case(sp, Q, K, V, dO, stripe, block, dtype)
    empty_row = np.ones((nb, nb), dtype=np.uint8)
    empty_row[2, :] = 0                                      # a block row with no kept block
    _run_attention_case(sp, Q, K, V, dO, empty_row, block, dtype)
    one = np.ones((1, 1), dtype=np.uint8)                    # smallest problem: L == block
    _run_attention_case(sp, Q[:, :block], K[:, :block], V[:, :block], dO[:, :block], one, block, dtype)
    none = np.zeros((nb, nb), dtype=np.uint8)                # nothing kept: zeros and -inf everywhere
    _run_attention_case(sp, Q, K, V, dO, none, block, dtype)


@pytest.mark.parametrize("block", [32, 64])
def test_attention_rows_without_a_diagonal_block(sp, block):
    # the bf16 row-walking kernels load the diagonal block early and visit it first; rows that do not
    # keep it take another path, and so do rows whose diagonal entry lies beyond the first 64 entries
    nb, BH, d = 6, 2, 64
    L = nb * block
    rng = np.random.default_rng(17 + block)
    Q, K, V, dO = [si.round_to_dtype(rng.standard_normal((BH, L, d), dtype=np.float32), "bf16")
                   for _ in range(4)]
    fl = si.random_block_mask(nb, 0.5, seed=block + 1)
    fl[np.arange(nb), np.arange(nb)] = 0                     # no row keeps its diagonal block
    fl[0, :] = 0
    fl[0, nb - 1] = 1                                        # single off-diagonal block
    fl[3, :] = 0                                             # empty row
    _run_attention_case(sp, Q, K, V, dO, fl, block, "bf16")
    anti = np.fliplr(np.eye(nb, dtype=np.uint8))             # anti-diagonal only
    _run_attention_case(sp, Q, K, V, dO, anti, block, "bf16")


def test_attention_long_rows_find_their_diagonal(sp):
    block, nb, BH, d = 32, 72, 1, 64                         # rows with more than 64 kept blocks
    L = nb * block
    rng = np.random.default_rng(23)
    Q, K, V, dO = [si.round_to_dtype(rng.standard_normal((BH, L, d), dtype=np.float32), "bf16")
                   for _ in range(4)]
    fl = np.eye(nb, dtype=np.uint8)
    fl[70, :] = 1                                            # diagonal entry at position 70
    fl[68, :] = 1
    fl[68, 68] = 0                                           # 71 entries, none of them the diagonal
    fl[5, :] = 1                                             # diagonal entry at position 5
    _run_attention_case(sp, Q, K, V, dO, fl, block, "bf16")


@pytest.mark.parametrize("dtype,block", [("bf16", 32), ("f32", 16)])
def test_attention_at_the_largest_block_grid(sp, dtype, block):
    """nb = 1024 (L = 32768 at block 32, 16384 at block 16): a key block kept by every block row (64 key-side chunks),
    a 120-row column, a 200-block row and a row without its diagonal block.  The dense oracle is out
    of reach at this size, so the check is on sampled outputs: the oracle gives the probabilities of
    one row at a time; O, LSE and dQ of sampled rows and dK, dV of sampled keys follow from them
    with the gradient formulas of Eq. 5.  dO is zero except on two rows of every block row (and the
    sampled rows): a row with dO = 0 adds nothing to dK, dV, so only those rows need the oracle,
    while every chunk of every split column still carries a non-zero share."""
    import os
    from concurrent.futures import ThreadPoolExecutor
    nb, d, BH, bh = 1024, 64, 2, 1
    L = nb * block
    scale = 1.0 / np.sqrt(d)
    rng = np.random.default_rng(77)
    fl = np.zeros((nb, nb), dtype=np.uint8)
    I = np.arange(nb)
    fl[I, I] = 1
    fl[I[1:], I[:-1]] = 1
    fl[I[:-1], I[1:]] = 1
    fl[:, 700] = 1
    fl[300:420, 77] = 1
    fl[513, rng.choice(nb, 200, replace=False)] = 1
    fl[900, 900] = 0
    Q, K, V, dO = [si.round_to_dtype(rng.standard_normal((BH, L, d), dtype=np.float32), dtype)
                   for _ in range(4)]
    rows = sorted({0, block - 1, block, 513 * block + 5, 514 * block - 1, 900 * block + 3, 77 * block, L - 1}
                  | set(rng.integers(0, L, 16).tolist()))
    live = sorted(set(rows) | set((I * block + I % block).tolist())
                  | set((I * block + (7 * I + 3) % block).tolist()))       # rows with dO != 0
    dead = np.ones(L, dtype=bool)
    dead[live] = False
    dO[:, dead, :] = 0.0
    pat = _pattern_from_mask(sp, fl, block)
    q, k, v, do = [_dev(t, _torch_dtype(dtype)).view(1, BH, L, d) for t in (Q, K, V, dO)]
    O, LSE = sp.attn_fwd(q, k, v, pat)
    dQ, dK, dV = sp.attn_bwd(q, k, v, O, do, LSE, pat)
    torch.cuda.synchronize()
    got = {n: t.float().cpu().numpy().reshape(BH, L, d)[bh] for n, t in
           (("O", O), ("dQ", dQ), ("dK", dK), ("dV", dV))}
    lse = LSE.cpu().numpy().reshape(BH, L)[bh]
    for x in got.values():
        assert np.all(np.isfinite(x))

    assert not got["dQ"][dead].any()                                   # dO = 0 rows: dS = 0 exactly
    P = np.repeat(np.repeat(fl, block, axis=0), block, axis=1)         # the mask, element by element
    Q64, K64, V64, dO64 = [np.ascontiguousarray(t, dtype=np.float64) for t in (Q, K, V, dO)]
    keys = np.array([700 * block + 1, 701 * block - 2, 77 * block + 7, 77 * block + block // 2, 5, L - 2])
    Vk, n_keys = V64[bh][keys], len(keys)

    def one_row(i):
        p = oracle.attn_probs_row(Q64, K64, P, bh, i)
        o = p @ V64[bh]
        delta = dO64[bh, i] @ o
        ds_k = p[keys] * (Vk @ dO64[bh, i] - delta)
        out = [np.outer(p[keys], dO64[bh, i]), scale * np.outer(ds_k, Q64[bh, i])]
        if i in rows:
            ds = p * (V64[bh] @ dO64[bh, i] - delta)
            j = int(np.argmax(p))
            out += [o, scale * (ds @ K64[bh]), scale * (Q64[bh, i] @ K64[bh, j]) - np.log(p[j])]
        return out

    rdV, rdK = np.zeros((n_keys, d)), np.zeros((n_keys, d))
    rO, rdQ, rLSE = {}, {}, {}
    with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as pool:
        for i, out in zip(live, pool.map(one_row, live, chunksize=16)):
            rdV += out[0]
            rdK += out[1]
            if len(out) > 2:
                rO[i], rdQ[i], rLSE[i] = out[2], out[3], out[4]
    tol = TOL[dtype]
    checks = {"O": (got["O"][rows], np.stack([rO[i] for i in rows])),
              "dQ": (got["dQ"][rows], np.stack([rdQ[i] for i in rows])),
              "dK": (got["dK"][keys], rdK), "dV": (got["dV"][keys], rdV)}
    for name, (x, ref) in checks.items():
        fro, mx = _rel_errors(x, ref)
        assert fro <= tol and mx <= tol, (name, fro, mx)
    ref_lse = np.array([rLSE[i] for i in rows])
    assert np.abs(lse[rows] - ref_lse).max() <= tol * max(np.abs(ref_lse).max(), 1.0)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_attention_tall_columns_are_split_into_chunks(sp, dtype):
    # columns with more kept rows than one key-side work item takes (16): 36, 25, 21 and 17 rows,
    # next to one with exactly 16
    block, nb, BH, d = 16, 36, 2, 64
    L = nb * block
    rng = np.random.default_rng(11)
    Q, K, V, dO = [si.round_to_dtype(rng.standard_normal((BH, L, d), dtype=np.float32), dtype)
                   for _ in range(4)]
    fl = np.eye(nb, dtype=np.uint8)
    fl[:, 4] = 1
    fl[:25, 9] = 1
    fl[15:, 15] = 1
    fl[14:31, 30] = 1
    fl[2:17, 33] = 1
    fl[3, :] = 1
    _run_attention_case(sp, Q, K, V, dO, fl, block, dtype)
    if dtype == "bf16":
        # the same columns at block 32: the tuned kernels, where every workgroup derives its chunk from
        # col_ptr and the partial tiles are added by a second launch
        Q2, K2, V2, dO2 = [si.round_to_dtype(rng.standard_normal((BH, nb * 32, d), dtype=np.float32), dtype)
                           for _ in range(4)]
        _run_attention_case(sp, Q2, K2, V2, dO2, fl, 32, dtype)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("block", [16, 32, 64])
def test_attention_paper_denominator_and_explicit_scale(sp, dtype, block):
    """Algorithm 6's denominator (every masked entry of a row counted as a score of 0) and an explicit
    scale, on every kernel family: block 32 / 64 in bf16 take the tuned kernels, the rest the generic
    ones.  The mask has a row without its diagonal block, a row that keeps a single off-diagonal
    block, a full row and a row that keeps nothing."""
    nb, BH, d = 6, 2, 64
    L = nb * block
    rng = np.random.default_rng(4 + block)
    Q, K, V, dO = [si.round_to_dtype(rng.standard_normal((BH, L, d), dtype=np.float32), dtype)
                   for _ in range(4)]
    fl = si.random_block_mask(nb, 0.4, seed=9)
    fl[1, 1] = 0
    fl[1, 4] = 1                                             # row 1: no diagonal block
    fl[2, :] = 0
    fl[2, 5] = 1                                             # row 2: one off-diagonal block
    fl[3, :] = 1                                             # row 3: nothing masked (both sums agree)
    fl[4, :] = 0                                             # row 4: nothing kept
    _run_attention_case(sp, Q, K, V, dO, fl, block, dtype, flags=sp.SPION_ATTN_PAPER_DENOM)
    _run_attention_case(sp, Q, K, V, dO, fl, block, dtype, scale=0.2)
    _run_attention_case(sp, Q, K, V, dO, fl, block, dtype, flags=sp.SPION_ATTN_PAPER_DENOM, scale=0.07)
    if dtype == "bf16":
        # scores of a few hundred: the kept maximum is far above the masked entries' 0.  (bf16 only: an
        # fp32 score of 300 carries a rounding error of 300 * 2^-24 = 2e-5 into the exponent, so the
        # 1e-5 bar of the fp32 path is not defined for such inputs.)
        big = [si.round_to_dtype(t * s_, dtype) for t, s_ in zip((Q, K, V, dO), (6.0, 6.0, 1.0, 1.0))]
        _run_attention_case(sp, *big, fl, block, dtype, flags=sp.SPION_ATTN_PAPER_DENOM)
    # every kept score negative (around -5): the row maximum lies below the masked entries' 0
    _run_attention_case(sp, np.abs(Q), -np.abs(K), V, dO, fl, block, dtype, flags=sp.SPION_ATTN_PAPER_DENOM)


def test_attention_large_scores_stay_finite(sp):
    block, nb, BH, d = 32, 3, 1, 64
    L = nb * block
    rng = np.random.default_rng(5)
    Q, K, V, dO = [si.round_to_dtype(rng.standard_normal((BH, L, d), dtype=np.float32) * s, "bf16")
                   for s in (6.0, 6.0, 1.0, 1.0)]          # scores of a few hundred
    fl = si.random_block_mask(nb, 0.6, seed=1)
    _run_attention_case(sp, Q, K, V, dO, fl, block, "bf16")


@pytest.mark.parametrize("name,heads", [("cfg1_tiny_f32_L256", None), ("cfg2_bf16_L1024", 16),
                                        ("cfg3_bf16_L2048", 8), ("cfg4_bf16_L4096", 4),
                                        ("cfg5_layer0", 2), ("cfg5_layer1", 2), ("cfg5_layer2", 2),
                                        ("cfg5_layer3", 2)])
def test_attention_workloads_full_size(sp, name, heads):
    """Full-size launch (all batch items and heads, the configuration the benchmark times) with the
    pattern spion_pattern produces from the mean over all (batch, head) slices, i.e. the benchmark's
    own index; the oracle checks a spread of (batch, head) slices."""
    w = si.workload(name)
    Q, K, V, dO, A = _workload_inputs(name)
    pat = sp.generate_pattern(_dev(A), w.block, w.filt, w.thresh_mode, w.thresh_value)
    fl = pat.fl_out.cpu().numpy()
    assert np.array_equal(fl, oracle.generate_pattern(A, w.block, w.filt, w.thresh_mode, w.thresh_value)["fl_out"])
    assert pat.nnzb == si.EXPECTED_NNZB[name]
    BH = w.B * w.H
    sel = None if heads is None else sorted(set(np.linspace(0, BH - 1, heads).astype(int).tolist()))
    errs = _run_attention_case(sp, Q, K, V, dO, fl, w.block, w.dtype, heads=sel)
    print(name, f"nnzb={pat.nnzb}", {k: f"{v[0]:.2e}/{v[1]:.2e}" for k, v in errs.items()})


def test_autograd_wrapper_matches_torch_masked_attention(sp):
    # the autograd front end against plain fp32 torch ops on the GPU (dense masked attention)
    block, nb, B, H, d = 32, 6, 2, 2, 64
    L = nb * block
    torch.manual_seed(0)
    fl = si.random_block_mask(nb, 0.4, seed=4)
    pat = _pattern_from_mask(sp, fl, block)
    q, k, v = [torch.randn(B, H, L, d, device="cuda", requires_grad=True) for _ in range(3)]
    do = torch.randn(B, H, L, d, device="cuda")
    o = sp.sparse_attention(q, k, v, pat)
    o.backward(do)
    got = [o.detach(), q.grad.clone(), k.grad.clone(), v.grad.clone()]
    for t in (q, k, v):
        t.grad = None
    P = torch.from_numpy(oracle.upsample(fl, block)).cuda().bool()
    s = (q @ k.transpose(-1, -2)) / 8.0
    ref = torch.softmax(s.masked_fill(~P, float("-inf")), dim=-1) @ v
    ref.backward(do)
    for g, r in zip(got, [ref.detach(), q.grad, k.grad, v.grad]):
        err = (g - r).norm() / r.norm()
        assert err < 5e-5, float(err)     # torch's own fp32 matmuls are the looser side here


@pytest.mark.parametrize("tdt", [torch.float32, torch.bfloat16])
def test_sparse_mha_sublayer_matches_plain_torch(sp, tdt):
    # Algorithm 5 as a module (LayerNorm, projections, heads, W^O, residual) against the same
    # sub-layer written with dense masked attention in plain torch ops, forward and all gradients
    block, nb, B, H = 32, 4, 2, 2
    L, D = nb * block, 64 * H
    torch.manual_seed(1)
    fl = si.random_block_mask(nb, 0.5, seed=7)
    pat = _pattern_from_mask(sp, fl, block)
    mha = sp.SparseMHA(D, H, dropout=0.0, device="cuda", dtype=tdt)
    E = torch.randn(B, L, D, device="cuda", dtype=tdt, requires_grad=True)
    dOut = torch.randn(B, L, D, device="cuda", dtype=tdt)
    out = mha(E, pat)
    out.backward(dOut)
    got = [out.detach().float(), E.grad.float().clone()] + [p.grad.float().clone() for p in mha.parameters()]
    E.grad = None
    mha.zero_grad()

    P = torch.from_numpy(oracle.upsample(fl, block)).cuda().bool()
    X = mha.norm(E)
    qkv = mha.w_qkv(X).view(B, L, 3, H, 64)
    q, k, v = [qkv[:, :, i].transpose(1, 2).float() for i in range(3)]
    a = torch.softmax((q @ k.transpose(-1, -2) / 8.0).masked_fill(~P, float("-inf")), dim=-1) @ v
    ref_out = mha.w_o(a.to(tdt).transpose(1, 2).reshape(B, L, D)) + E
    ref_out.backward(dOut)
    ref = [ref_out.detach().float(), E.grad.float()] + [p.grad.float() for p in mha.parameters()]
    tol = 1e-4 if tdt == torch.float32 else 3e-2
    for g, r in zip(got, ref):
        assert torch.isfinite(g).all()
        assert float((g - r).norm() / r.norm()) < tol
    mha.train()
    drop = sp.SparseMHA(D, H, dropout=0.5, device="cuda", dtype=tdt)
    assert drop(E.detach(), pat).shape == (B, L, D)


def test_attention_backward_is_deterministic(sp):
    w = si.workload(2)
    Q, K, V, dO = si.make_qkv_do(w, bh_limit=8)
    fl = si.random_block_mask(w.nb, 0.2, seed=2)
    fl[:, 3] = 1
    pat = _pattern_from_mask(sp, fl, w.block)
    q, k, v, do = [_dev(t, torch.bfloat16).view(2, 4, w.L, w.d) for t in (Q, K, V, dO)]
    O, LSE = sp.attn_fwd(q, k, v, pat)
    first = [t.clone() for t in sp.attn_bwd(q, k, v, O, do, LSE, pat)]
    for _ in range(3):
        again = sp.attn_bwd(q, k, v, O, do, LSE, pat)
        for a, b in zip(first, again):
            assert torch.equal(a, b)


def test_backward_phases_run_separately_give_the_same_bits(sp):
    # the two phase flags (used for per-phase timing): query side, then key side on the same
    # workspace, against the one-call backward
    w = si.workload(2)
    Q, K, V, dO = si.make_qkv_do(w, bh_limit=8)
    A = si.make_score_map(w, Q, K)
    pat = sp.generate_pattern(_dev(A), w.block, w.filt, w.thresh_mode, w.thresh_value)
    q, k, v, do = [_dev(t, torch.bfloat16).view(2, 4, w.L, w.d) for t in (Q, K, V, dO)]
    O, LSE = sp.attn_fwd(q, k, v, pat)
    ref = sp.attn_bwd(q, k, v, O, do, LSE, pat)
    code = sp.SPION_BF16
    ws = torch.empty(sp.spion_attn_workspace_bytes(2, 4, w.L, w.d, w.block, code, pat.nnzb, True),
                     dtype=torch.uint8, device="cuda")
    got = [torch.full_like(q, float("nan")) for _ in range(3)]
    for flags in (sp.SPION_ATTN_BWD_QUERY_SIDE_ONLY, sp.SPION_ATTN_BWD_KEY_SIDE_ONLY):
        sp.spion_attn_bwd(q, k, v, O, do, LSE, got[0], got[1], got[2], pat.row_ptr, pat.col_idx,
                          pat.col_ptr, pat.row_idx, pat.bsr_pos, pat.nnzb, 2, 4, w.L, w.d, w.block, code,
                          flags=flags, workspace=ws)
    torch.cuda.synchronize()
    for g, r in zip(got, ref):
        assert torch.equal(g, r)


def test_index_check_accepts_generated_patterns_and_flags_malformed_ones(sp):
    """spion_index_check against the oracle's compaction: the oracle's index of a random mask passes;
    each single corruption of it (every one still safe to read: the checker looks at an entry only
    after the stage before has shown its position to be in range) is reported."""
    w = si.workload(2)
    Q, K, _, _ = si.make_qkv_do(w, bh_limit=4)
    pat = sp.generate_pattern(_dev(si.make_score_map(w, Q, K)), w.block, w.filt, w.thresh_mode, w.thresh_value)
    assert sp.index_is_well_formed(pat)

    nb = 40
    fl = si.random_block_mask(nb, 0.3, seed=9)
    good = _pattern_from_mask(sp, fl, 16)
    assert sp.index_is_well_formed(good)
    bsr_only = _pattern_from_mask(sp, fl, 16)
    bsr_only.col_ptr = bsr_only.row_idx = bsr_only.bsr_pos = None
    assert sp.index_is_well_formed(bsr_only)
    empty = _pattern_from_mask(sp, np.zeros((nb, nb), dtype=np.uint8), 16)
    assert sp.index_is_well_formed(empty)

    c = oracle.compact(fl)
    n = c["nnzb"]
    r5 = int(c["row_ptr"][5])
    assert c["row_ptr"][6] - r5 >= 2 and c["col_ptr"][4] - c["col_ptr"][3] >= 2

    def corrupt(field, index, value):
        bad = _pattern_from_mask(sp, fl, 16)
        getattr(bad, field)[index] = value
        return bad

    cases = {
        "row_ptr decreases": corrupt("row_ptr", 7, int(c["row_ptr"][6]) - 1),
        "row_ptr does not start at 0": corrupt("row_ptr", 0, 1),
        "row_ptr beyond nnzb": corrupt("row_ptr", nb, n + 3),
        "column out of range": corrupt("col_idx", r5, nb),
        "negative column": corrupt("col_idx", r5, -1),
        "columns not ascending": corrupt("col_idx", r5 + 1, int(c["col_idx"][r5])),
        "col_ptr decreases": corrupt("col_ptr", 3, int(c["col_ptr"][4]) + 1),
        "row out of range": corrupt("row_idx", int(c["col_ptr"][3]), nb + 5),
        "bsr_pos out of range": corrupt("bsr_pos", 0, n),
        "bsr_pos names another block": corrupt("bsr_pos", int(c["col_ptr"][3]), int(c["bsr_pos"][c["col_ptr"][3] + 1])),
    }
    for what, bad in cases.items():
        assert not sp.index_is_well_formed(bad), what
    wrong_count = _pattern_from_mask(sp, fl, 16)
    wrong_count.nnzb = n - 1
    assert not sp.index_is_well_formed(wrong_count)


def test_step_and_pattern_replay_from_hip_graphs(sp):
    """The library enqueues kernels only (no allocation, no memset, no synchronisation), so a
    forward + backward step and a pattern generation can be captured into HIP graphs.  Every replay,
    with eager work and synchronisations in between and with new contents in the captured buffers,
    must give the bits of the eager calls."""
    w = si.workload(2)
    B, H = 2, 4
    code = sp.SPION_BF16
    sets = []
    for off in (0, 1):
        Q, K, V, dO = si.make_qkv_do(w, seed_offset=off, bh_limit=B * H)
        sets.append([_dev(t, torch.bfloat16).view(B, H, w.L, w.d) for t in (Q, K, V, dO)])
    A = [_dev(si.make_score_map(w, Q, K, seed_offset=off)) for off in (0, 1)]
    pat = sp.generate_pattern(A[0], w.block, w.filt, w.thresh_mode, w.thresh_value)
    nnzb = pat.nnzb

    def eager(qkvdo):
        O, LSE = sp.attn_fwd(*qkvdo[:3], pat)
        return [O, LSE] + list(sp.attn_bwd(*qkvdo[:3], O, qkvdo[3], LSE, pat))

    want = [[t.clone() for t in eager(s_)] for s_ in sets]
    want_pat = []
    for a in A:
        p_ = sp.generate_pattern(a, w.block, w.filt, w.thresh_mode, w.thresh_value)
        want_pat.append((p_.fl_out.clone(), p_.col_idx[:p_.nnzb].clone(), p_.nnzb))

    # static buffers of the captured step
    q, k, v, do = [torch.empty_like(t) for t in sets[0]]
    O, dQ, dK, dV = [torch.empty_like(q) for _ in range(4)]
    LSE = torch.empty((B, H, w.L), dtype=torch.float32, device="cuda")
    ws = torch.empty(sp.spion_attn_workspace_bytes(B, H, w.L, w.d, w.block, code, nnzb, True),
                     dtype=torch.uint8, device="cuda")
    a_static = torch.empty_like(A[0])
    pat_static = sp.generate_pattern(A[0], w.block, w.filt, w.thresh_mode, w.thresh_value)
    ws_pat = torch.empty(sp.spion_pattern_workspace_bytes(w.L, w.block), dtype=torch.uint8, device="cuda")

    def step():
        sp.spion_attn_fwd(q, k, v, O, LSE, pat.row_ptr, pat.col_idx, nnzb, B, H, w.L, w.d, w.block, code)
        sp.spion_attn_bwd(q, k, v, O, do, LSE, dQ, dK, dV, pat.row_ptr, pat.col_idx, pat.col_ptr,
                          pat.row_idx, pat.bsr_pos, nnzb, B, H, w.L, w.d, w.block, code, workspace=ws)

    def regen():
        sp.generate_pattern(a_static, w.block, w.filt, w.thresh_mode, w.thresh_value, sync=False,
                            out=pat_static, workspace=ws_pat)

    for t, src in zip((q, k, v, do), sets[0]):
        t.copy_(src)
    a_static.copy_(A[0])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
        regen()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g_step, g_pat = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
    with torch.cuda.graph(g_step):
        step()
    with torch.cuda.graph(g_pat):
        regen()

    for which in (0, 1, 0, 1, 1):
        for t, src in zip((q, k, v, do), sets[which]):
            t.copy_(src)
        a_static.copy_(A[which])
        for t in (O, dQ, dK, dV, LSE):
            t.fill_(float("nan"))
        g_step.replay()
        g_pat.replay()
        torch.cuda.synchronize()
        for got, ref in zip((O, LSE, dQ, dK, dV), want[which]):
            assert torch.equal(got, ref)
        fl_ref, col_ref, n_ref = want_pat[which]
        assert int(pat_static.nnzb_dev.item()) == n_ref
        assert torch.equal(pat_static.fl_out, fl_ref) and torch.equal(pat_static.col_idx[:n_ref], col_ref)
        eager(sets[1 - which])                      # the program's own eager work between replays
        torch.cuda.synchronize()


def test_error_codes_need_no_launch(sp):
    A = torch.zeros((64, 64), device="cuda")
    with pytest.raises(sp.SpionError) as e:
        sp.generate_pattern(A, 16, 4, si.T_QUANTILE, 0.5)          # even filter
    assert e.value.code == -5
    with pytest.raises(sp.SpionError) as e:
        sp.generate_pattern(A, 24, 5, si.T_QUANTILE, 0.5)          # unsupported block
    assert e.value.code == -2
    with pytest.raises(sp.SpionError) as e:
        sp.generate_pattern(A, 16, 5, si.T_QUANTILE, 1.5)          # quantile outside [0, 1]
    assert e.value.code == -5
