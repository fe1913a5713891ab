"""Pins for the pattern half of the CPU oracle (no GPU needed).

Each step of Algorithm 3 is checked against something other than the oracle itself: closed forms,
numpy / scipy routines, hand-traced walk-throughs and brute-force reachability.
"""
import itertools
import os

import numpy as np
import pytest
import scipy.signal

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
ONE = 1 << 40


# ------------------------------------------------------------------ quantisation
def test_quantize_exact_values_and_ties_to_even():
    a = np.array([0.0, 1.0, 0.5, -0.25, 1.5 / ONE, 2.5 / ONE, 3.5 / ONE, -2.5 / ONE, 0.75 / ONE],
                 dtype=np.float32)
    q = oracle.quantize(a)
    assert q.tolist() == [0, ONE, ONE // 2, -(ONE // 4), 2, 2, 4, -2, 1]


def test_quantize_is_exact_for_ordinary_floats():
    rng = np.random.default_rng(0)
    a = rng.random(1000, dtype=np.float32) + np.float32(2.0 ** -10)   # >= 2^-10: 2^40*a is an integer
    q = oracle.quantize(a)
    assert np.array_equal(q.astype(np.float64), a.astype(np.float64) * ONE)


# ------------------------------------------------------------------ Eq. 3
@pytest.mark.parametrize("L,F", [(8, 3), (12, 5), (9, 7), (16, 31)])
def test_conv_delta_gives_clipped_diagonal_segment(L, F):
    p = (F - 1) // 2
    for (r, s) in [(0, 0), (L - 1, L - 1), (2, 5), (L // 2, 1), (0, L - 1)]:
        a = np.zeros((L, L), dtype=np.int64)
        a[r, s] = 7
        out = oracle.conv_diag(a, F)
        exp = np.zeros_like(a)
        for f in range(-p, p + 1):
            i, j = r + f, s + f
            if 0 <= i < L and 0 <= j < L:
                exp[i, j] = 7
        assert np.array_equal(out, exp)


@pytest.mark.parametrize("L,F", [(10, 1), (10, 5), (7, 9), (20, 31)])
def test_conv_identity_and_constant_closed_forms(L, F):
    p = (F - 1) // 2
    out = oracle.conv_diag(np.eye(L, dtype=np.int64), F)
    i = np.arange(L)
    assert np.array_equal(np.diag(out), np.minimum(i, p) + np.minimum(L - 1 - i, p) + 1)
    assert np.count_nonzero(out - np.diag(np.diag(out))) == 0
    c = 3
    out = oracle.conv_diag(np.full((L, L), c, dtype=np.int64), F)
    ii, jj = np.meshgrid(i, i, indexing="ij")
    exp = c * (np.minimum(np.minimum(ii, jj), p) + np.minimum(np.minimum(L - 1 - ii, L - 1 - jj), p) + 1)
    assert np.array_equal(out, exp)


def test_conv_filter_size_one_is_identity():
    rng = np.random.default_rng(1)
    a = rng.integers(-50, 50, size=(11, 11))
    assert np.array_equal(oracle.conv_diag(a, 1), a)


@pytest.mark.parametrize("L,F", [(13, 3), (16, 5), (24, 31), (9, 9)])
def test_conv_matches_scipy_correlate_with_identity_filter(L, F):
    rng = np.random.default_rng(L * 100 + F)
    a = rng.integers(-1000, 1000, size=(L, L)).astype(np.int64)
    ref = scipy.signal.correlate2d(a, np.eye(F, dtype=np.int64), mode="same", boundary="fill", fillvalue=0)
    assert np.array_equal(oracle.conv_diag(a, F), ref)


def test_conv_is_not_symmetric_under_transposed_filter():
    # an anti-diagonal filter would give a different answer: guards against a flipped index
    a = np.zeros((6, 6), dtype=np.int64)
    a[1, 4] = 1
    out = oracle.conv_diag(a, 3)
    assert out[0, 3] == 1 and out[2, 5] == 1 and out[0, 5] == 0 and out[2, 3] == 0


# ------------------------------------------------------------------ Eq. 4
@pytest.mark.parametrize("L,bs", [(8, 2), (12, 4), (16, 16), (6, 1)])
def test_pool_matches_reshape_sum_and_preserves_total(L, bs):
    rng = np.random.default_rng(L + bs)
    c = rng.integers(-10**6, 10**6, size=(L, L)).astype(np.int64)
    ps = oracle.pool_sum(c, bs)
    nb = L // bs
    assert np.array_equal(ps, c.reshape(nb, bs, nb, bs).sum(axis=(1, 3)))
    assert ps.sum() == c.sum()


def test_pool_rows_and_columns_not_swapped():
    c = np.zeros((4, 4), dtype=np.int64)
    c[0, 3] = 5          # row block 0, column block 1
    assert oracle.pool_sum(c, 2).tolist() == [[0, 5], [0, 0]]


# ------------------------------------------------------------------ threshold
def test_quantile_nearest_rank_matches_numpy_lower():
    rng = np.random.default_rng(5)
    for nb in (2, 3, 5, 8):
        ps = rng.integers(-10**12, 10**12, size=(nb, nb)).astype(np.int64)
        for q in (0.0, 0.1, 0.5, 0.85, 0.96, 0.99, 1.0):
            t = oracle.threshold(ps, 4, oracle.T_QUANTILE, q)
            k = int(np.floor(q * (nb * nb - 1)))
            assert t.is_int == 1 and t.ti == np.sort(ps.ravel())[k]
            assert t.ti == int(np.quantile(ps.ravel().astype(np.float64), q, method="lower"))


def test_quantile_hand_cases():
    ps = np.array([[10, 40], [30, 20]], dtype=np.int64)
    assert oracle.threshold(ps, 1, oracle.T_QUANTILE, 0.0).ti == 10
    assert oracle.threshold(ps, 1, oracle.T_QUANTILE, 0.34).ti == 20     # floor(0.34*3) = 1
    assert oracle.threshold(ps, 1, oracle.T_QUANTILE, 0.67).ti == 30     # floor(2.01) = 2
    assert oracle.threshold(ps, 1, oracle.T_QUANTILE, 1.0).ti == 40
    # values beyond 2^53 stay exact (no trip through double)
    big = np.array([[2**60 + 1, 2**60 + 3], [2**60 + 2, 2**60]], dtype=np.int64)
    assert oracle.threshold(big, 1, oracle.T_QUANTILE, 0.5).ti == 2**60 + 1


def test_mean_kstd_hand_case_and_numpy():
    ps = np.array([[2, 4], [4, 6]], dtype=np.int64)      # mean 4, population var 2
    t = oracle.threshold(ps, 1, oracle.T_MEAN_KSTD, 1.0)
    assert t.is_int == 0 and t.td == 4.0 + np.sqrt(2.0)
    t = oracle.threshold(ps, 1, oracle.T_MEAN_KSTD, -2.0)
    assert t.td == 4.0 - 2.0 * np.sqrt(2.0)
    rng = np.random.default_rng(9)
    ps = rng.integers(0, 10**15, size=(16, 16)).astype(np.int64)
    t = oracle.threshold(ps, 16, oracle.T_MEAN_KSTD, 1.0)
    x = ps.astype(np.float64)
    assert t.td == pytest.approx(x.mean() + x.std(), rel=1e-13)


def test_absolute_threshold_is_in_pool_out_units():
    ps = np.zeros((2, 2), dtype=np.int64)
    t = oracle.threshold(ps, 4, oracle.T_ABS, 0.5)
    assert t.is_int == 0 and t.td == 0.5 * 16 * ONE


# ------------------------------------------------------------------ Algorithm 4 + Algorithm 3
def _load_walkthroughs():
    cases, cur = [], None
    with open(os.path.join(GOLDEN, "flood_fill_hand_traced.txt")) as fh:
        rows = []
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if line.startswith("case"):
                if cur:
                    cur["fl"] = rows
                    cases.append(cur)
                cur, rows = {"name": line.split()[1]}, []
            elif line.startswith("t "):
                cur["t"] = int(line.split()[1])
            elif line == "=>":
                cur["pool"], rows = rows, []
            else:
                rows.append([int(v) for v in line.split()])
        cur["fl"] = rows
        cases.append(cur)
    return cases


@pytest.mark.parametrize("case", _load_walkthroughs(), ids=lambda c: c["name"])
def test_fill_hand_traced_walkthroughs(case):
    ps = np.array(case["pool"], dtype=np.int64)
    fl = oracle.fill(ps, oracle.make_thresh_int(case["t"]))
    assert fl.tolist() == case["fl"]


def brute_force_fill(x: np.ndarray, t, force_diag=True) -> np.ndarray:
    """Reachability over the 'neighbours equal to their maximum' successor relation, written
    independently of the oracle's walks: breadth-first over Python sets from every seed; reached
    cells above t are kept."""
    nb = x.shape[0]

    def succ(r, c):
        if r + 1 == nb or c + 1 == nb:
            return []
        cand = [(r + 1, c), (r, c + 1), (r + 1, c + 1)]
        m = max(x[a, b] for a, b in cand)
        return [(a, b) for a, b in cand if x[a, b] == m]

    seeds = [(0, i) for i in range(nb)] + [(j, 0) for j in range(nb)]
    reached, frontier = set(), []
    for s in seeds:
        frontier.extend(succ(*s))
    while frontier:
        cell = frontier.pop()
        if cell in reached:
            continue
        reached.add(cell)
        frontier.extend(succ(*cell))
    fl = np.zeros((nb, nb), dtype=np.uint8)
    for (a, b) in reached:
        if x[a, b] > t:
            fl[a, b] = 1
    if force_diag:
        fl[np.arange(nb), np.arange(nb)] = 1
    return fl


def test_fill_equals_brute_force_on_all_3x3_maps_with_ties():
    for vals in itertools.product(range(3), repeat=9):
        x = np.array(vals, dtype=np.int64).reshape(3, 3)
        for t in (-1, 0, 1):
            got = oracle.fill(x, oracle.make_thresh_int(t), force_diag=False)
            assert np.array_equal(got, brute_force_fill(x, t, force_diag=False)), (vals, t)


@pytest.mark.parametrize("nb", [2, 4, 5, 6, 9])
def test_fill_equals_brute_force_on_random_maps(nb):
    rng = np.random.default_rng(nb)
    for trial in range(200):
        hi = [2, 3, 10, 1000][trial % 4]          # small ranges force ties and plateaus
        x = rng.integers(0, hi, size=(nb, nb)).astype(np.int64)
        t = int(rng.integers(-1, hi))
        got = oracle.fill(x, oracle.make_thresh_int(t))
        assert np.array_equal(got, brute_force_fill(x, t)), (x, t)


def test_fill_double_threshold_agrees_with_integer_threshold():
    rng = np.random.default_rng(77)
    x = rng.integers(0, 50, size=(7, 7)).astype(np.int64)
    a = oracle.fill(x, oracle.make_thresh_int(20))
    b = oracle.fill(x, oracle.make_thresh_double(20.0))
    c = oracle.fill(x, oracle.make_thresh_double(20.5))
    assert np.array_equal(a, b) and np.array_equal(a, c)


def test_fill_invariants():
    rng = np.random.default_rng(3)
    nb = 12
    x = rng.integers(0, 10**9, size=(nb, nb)).astype(np.int64)
    t = int(np.sort(x.ravel())[100])
    raw = oracle.fill(x, oracle.make_thresh_int(t), force_diag=False)
    assert raw[0, 0] == 0                                  # a seed is never marked by its own call
    assert np.all(x[raw == 1] > t)                         # every marked cell exceeds t
    fl = oracle.fill(x, oracle.make_thresh_int(t))
    assert np.all(np.diag(fl) == 1)
    assert np.array_equal(fl - np.diag(np.diag(fl)), raw - np.diag(np.diag(raw)))
    # constant map with t >= the constant marks nothing
    const = np.full((5, 5), 4, dtype=np.int64)
    assert oracle.fill(const, oracle.make_thresh_int(4), force_diag=False).sum() == 0
    # ... and with t below the constant marks everything reachable: all but row 0 / col 0 seeds'
    # own cells that nobody steps onto, i.e. everything except (0,0)
    full = oracle.fill(const, oracle.make_thresh_int(3), force_diag=False)
    exp = np.ones((5, 5), dtype=np.uint8)
    exp[0, 0] = 0
    assert np.array_equal(full, exp)


def test_fill_follows_a_dominant_column_and_a_dominant_diagonal():
    nb = 8
    x = np.ones((nb, nb), dtype=np.int64)
    x[:, 5] = 100
    fl = oracle.fill(x, oracle.make_thresh_int(50), force_diag=False)
    exp = np.zeros((nb, nb), dtype=np.uint8)
    exp[1:, 5] = 1                         # (0,5) is a seed: only cells stepped onto are marked
    exp[0, 5] = 1                          # ... but (0,4)'s right neighbour is (0,5)
    assert np.array_equal(fl, exp)
    x = np.arange(nb * nb, dtype=np.int64).reshape(nb, nb) % 7   # noise below the threshold
    x[np.arange(nb), np.arange(nb)] = 100
    fl = oracle.fill(x, oracle.make_thresh_int(50), force_diag=False)
    exp = np.eye(nb, dtype=np.uint8)
    exp[0, 0] = 0
    assert np.array_equal(fl, exp)


def test_fill_on_large_plateaus_is_linear_work():
    # all pooled values equal: every neighbour ties, a literal re-expansion of unmarked cells would
    # be exponential; everything except (0, 0) is reachable
    nb = 64
    const = np.zeros((nb, nb), dtype=np.int64)
    assert oracle.fill(const, oracle.make_thresh_int(5), force_diag=False).sum() == 0
    full = oracle.fill(const, oracle.make_thresh_int(-1), force_diag=False)
    assert full.sum() == nb * nb - 1 and full[0, 0] == 0


def fill_by_predecessors(x: np.ndarray, t, force_diag=True) -> np.ndarray:
    """The same set computed the other way round: moves only go down, right or down-right, so in
    row-major order every predecessor of a cell is settled before the cell.  A cell is stepped onto
    iff one of its three predecessors is a live cell (a seed of the first row / column, or itself
    stepped onto), lies outside the last row and column, and sees the cell among the largest of
    its own three neighbours."""
    nb = x.shape[0]
    live = np.zeros((nb, nb), dtype=bool)        # a walk stands on this cell at some point
    stepped = np.zeros((nb, nb), dtype=bool)
    live[0, :] = True
    live[:, 0] = True
    for r in range(nb):
        for c in range(nb):
            for pr, pc in ((r - 1, c), (r, c - 1), (r - 1, c - 1)):
                if pr < 0 or pc < 0 or not live[pr, pc] or pr == nb - 1 or pc == nb - 1:
                    continue
                if x[r, c] == max(x[pr + 1, pc], x[pr, pc + 1], x[pr + 1, pc + 1]):
                    stepped[r, c] = True
            live[r, c] |= stepped[r, c]
    fl = (stepped & (x > t)).astype(np.uint8)
    if force_diag:
        fl[np.arange(nb), np.arange(nb)] = 1
    return fl


@pytest.mark.parametrize("nb", [2, 3, 7, 16, 40])
def test_fill_equals_predecessor_sweep_on_random_maps(nb):
    rng = np.random.default_rng(100 + nb)
    for trial in range(60):
        hi = [2, 4, 50, 10**9][trial % 4]
        x = rng.integers(0, hi, size=(nb, nb)).astype(np.int64)
        t = int(rng.integers(-1, hi))
        assert np.array_equal(oracle.fill(x, oracle.make_thresh_int(t)), fill_by_predecessors(x, t)), (x, t)
        assert np.array_equal(brute_force_fill(x, t), fill_by_predecessors(x, t))


def test_topk_variant_keeps_blocks_above_threshold_plus_diagonal():
    x = np.array([[1, 9, 2], [8, 1, 1], [1, 1, 1]], dtype=np.int64)
    fl = oracle.topk(x, oracle.make_thresh_int(5))
    assert fl.tolist() == [[1, 1, 0], [1, 1, 0], [0, 0, 1]]


# ------------------------------------------------------------------ compaction / upsampling
def test_compact_invariants_and_transpose():
    rng = np.random.default_rng(11)
    for nb in (1, 2, 5, 16, 33):
        fl = (rng.random((nb, nb)) < 0.3).astype(np.uint8)
        fl[np.arange(nb), np.arange(nb)] = 1
        c = oracle.compact(fl)
        assert c["nnzb"] == int(fl.sum()) == c["row_ptr"][nb] == c["col_ptr"][nb]
        assert np.all(np.diff(c["row_ptr"]) >= 0)
        dense = np.zeros_like(fl)
        for I in range(nb):
            cols = c["col_idx"][c["row_ptr"][I]:c["row_ptr"][I + 1]]
            assert np.all(np.diff(cols) > 0)
            dense[I, cols] = 1
        assert np.array_equal(dense, fl)
        dense_t = np.zeros_like(fl)
        for J in range(nb):
            rows = c["row_idx"][c["col_ptr"][J]:c["col_ptr"][J + 1]]
            assert np.all(np.diff(rows) > 0)
            dense_t[rows, J] = 1
            for k in range(c["col_ptr"][J], c["col_ptr"][J + 1]):
                pos = c["bsr_pos"][k]
                I = c["row_idx"][k]
                assert c["col_idx"][pos] == J and c["row_ptr"][I] <= pos < c["row_ptr"][I + 1]
        assert np.array_equal(dense_t, fl)
        import scipy.sparse
        ref = scipy.sparse.csr_matrix(fl)
        ref.sort_indices()
        assert np.array_equal(ref.indptr, c["row_ptr"]) and np.array_equal(ref.indices, c["col_idx"])


def test_upsample_is_nearest_neighbour():
    fl = np.array([[1, 0], [0, 1]], dtype=np.uint8)
    P = oracle.upsample(fl, 3)
    assert np.array_equal(P, np.kron(fl, np.ones((3, 3), dtype=np.uint8)))


# ------------------------------------------------------------------ end to end on a planted map
def test_generate_pattern_finds_planted_band_on_tiny_workload():
    import spion_inputs as si
    w = si.workload(1)
    Q, K, V, dO = si.make_qkv_do(w)
    A = si.make_score_map(w, Q, K)
    out = oracle.generate_pattern(A, w.block, w.filt, w.thresh_mode, w.thresh_value)
    fl = out["fl_out"]
    assert np.all(np.diag(fl) == 1)
    assert 0.02 < fl.mean() < 0.6
    # pool_sum equals the direct float evaluation of Eq. 3 + Eq. 4 up to quantisation
    p = (w.filt - 1) // 2
    conv = np.zeros((w.L, w.L))
    for f in range(-p, p + 1):
        lo, hi = max(0, -f), min(w.L, w.L - f)
        conv[lo:hi, lo:hi] += A[lo + f:hi + f, lo + f:hi + f].astype(np.float64)
    ref = conv.reshape(w.nb, w.block, w.nb, w.block).sum(axis=(1, 3))
    assert np.allclose(out["pool_sum"] / ONE, ref, rtol=0, atol=w.block ** 2 * w.filt * 2.0 ** -40)


# ------------------------------------------------------------------ producers of the pattern input
def test_score_mean_matches_numpy_and_special_cases():
    rng = np.random.default_rng(21)
    maps = rng.random((5, 12, 12))
    assert np.allclose(oracle.score_mean(maps), maps.mean(axis=0), rtol=1e-15)
    assert np.array_equal(oracle.score_mean(maps[:1]), maps[0])            # one map: identity
    const = np.stack([np.full((4, 4), v) for v in (1.0, 2.0, 6.0)])
    assert np.array_equal(oracle.score_mean(const), np.full((4, 4), 3.0))
    # the mean is taken over maps, not over rows or columns
    two = np.zeros((2, 2, 2))
    two[0, 0, 1] = 4.0
    assert oracle.score_mean(two).tolist() == [[0.0, 2.0], [0.0, 0.0]]


def test_frobenius_distance_hand_case_and_numpy():
    a = np.array([[3.0, 0.0], [0.0, 4.0]])        # norm 5
    b = np.array([[5.0, 12.0], [0.0, 0.0]])       # norm 13
    d, na, nb_ = oracle.frobenius_distance(a, b)
    assert (d, na, nb_) == (8.0, 5.0, 13.0)
    assert oracle.frobenius_distance(b, a)[0] == 8.0                      # absolute value
    rng = np.random.default_rng(22)
    x, y = rng.standard_normal((2, 50, 50))
    d, nx, ny = oracle.frobenius_distance(x, y)
    assert nx == pytest.approx(np.linalg.norm(x), rel=1e-14) and ny == pytest.approx(np.linalg.norm(y), rel=1e-14)
    assert d == pytest.approx(abs(np.linalg.norm(x) - np.linalg.norm(y)), rel=1e-10)
    # Eq. 2 is the difference of the norms, not the norm of the difference
    assert oracle.frobenius_distance(a, -a)[0] == 0.0
