"""Pins of the CPU oracle against things other than itself: hand-worked values
of Equation 2, published SplitMix64 vectors, closed forms, brute-force dense
products, SciPy's CSR product and the sampler's invariants (Sections 4.2, 4.4,
5.3 of the paper).  No GPU needed."""
import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from workloads import make_workload, random_csr


# --------------------------------------------------------------------------
# sample index: golden values
# --------------------------------------------------------------------------
def _golden_rows(golden, name):
    for left, right in golden(name):
        seed, row, n, W = (int(t) for t in left)
        k = min(n, W)
        expect = list(range(k)) if right == ["@identity"] else [int(t) for t in right]
        assert len(expect) == k, (name, left)
        yield seed, row, n, W, expect


@pytest.mark.parametrize("name", ["fastrand_eq2.txt", "fastrand_rotation.txt"])
def test_fastrand_golden_values(golden, name):
    for seed, row, n, W, expect in _golden_rows(golden, name):
        got = [oracle.sample_index("fastrand", seed, row, i, n, W) for i in range(len(expect))]
        assert got == expect, (name, seed, row, n, W)
        # the row-list entry point must agree with the per-slot one: put the
        # row at index `row` of a graph whose other rows are empty
        rowptr = np.zeros(row + 2, dtype=np.int64)
        rowptr[row + 1:] = n
        if n < 2 ** 31:
            pos, cnt = oracle.kept(rowptr.astype(np.int32), W, "fastrand", seed, rows=[row])
            assert cnt[0] == len(expect)
            assert pos[0, :cnt[0]].tolist() == expect


def test_splitmix64_published_vectors(golden):
    for left, right in golden("splitmix64.txt"):
        seed = int(left[0])
        expect = [int(t) for t in right]
        assert oracle.splitmix64_stream(seed, len(expect)) == expect


def test_rotation_uses_high_word_of_row_plus_one(golden):
    (left, right), = [g for g in golden("splitmix64.txt") if g[0] == ["1234567"]]
    outs = [int(t) for t in right]
    for row, out in enumerate(outs):
        for n in (1000, 7, 2 ** 31 - 1):
            assert oracle.offset(1234567, row, n) == (out >> 32) % n
    assert oracle.offset(0, 5, 1000) == 0


def test_multiplier_rule():
    assert oracle.multiplier(1000) == 577
    assert oracle.multiplier(577) == 587
    assert oracle.multiplier(577 * 587) == 593
    assert oracle.multiplier(577 * 587 * 593) == 599
    assert oracle.multiplier(587) == 577
    for n in range(1, 4000):
        p = oracle.multiplier(n)
        assert p == (577 if n % 577 else 587)


# --------------------------------------------------------------------------
# sampler invariants
# --------------------------------------------------------------------------
def _single_row_rowptr(n):
    return np.array([0, n], dtype=np.int32)


def test_bucket_is_first_k_positions():
    rowptr, _ = random_csr(300, 9.0, seed=11, empty_frac=0.1)
    deg = np.diff(rowptr)
    for W in (1, 4, 9, 64):
        pos, cnt = oracle.kept(rowptr, W, "bucket", seed=99)
        assert (cnt == np.minimum(deg, W)).all()
        for r in range(300):
            k = cnt[r]
            assert (pos[r, :k] == rowptr[r] + np.arange(k)).all()
            assert (pos[r, k:] == -1).all()


def test_distinct_subset_exhaustive_small_n():
    """For every n <= 3000 and the hardest width W = n-1, FastRand keeps n-1
    distinct in-row positions (any smaller W is a prefix of that list)."""
    for seed in (0, 42):
        for n in range(2, 3001):
            pos, cnt = oracle.kept(_single_row_rowptr(n), n - 1, "fastrand", seed)
            p = pos[0]
            assert cnt[0] == n - 1
            assert p.min() >= 0 and p.max() < n
            assert np.unique(p).size == n - 1, n


def test_distinct_for_multiples_of_the_primes():
    ns = [577 * m for m in range(1, 120)] + [577 * 587 * m for m in (1, 2, 3, 5)]
    ns += [587 * m for m in (1, 2, 577)] + [577 * 587 * 593]
    for n in ns:
        W = min(n - 1, 4096)
        pos, cnt = oracle.kept(_single_row_rowptr(n), W, "fastrand", 0)
        assert cnt[0] == W
        assert np.unique(pos[0]).size == W, n
        assert pos[0].min() >= 0 and pos[0].max() < n


def test_prefix_property():
    """The list for width W is the first W slots of the list for any larger
    width, as long as both are below n (slot i never depends on W)."""
    n = 5000
    big, _ = oracle.kept(_single_row_rowptr(n), 512, "fastrand", 3)
    for W in (1, 16, 100, 511):
        small, _ = oracle.kept(_single_row_rowptr(n), W, "fastrand", 3)
        assert (small[0] == big[0, :W]).all()


def test_counts_match_sampling_rate_formula():
    """Section 5.3: the kept fraction is sum(min(deg, S)) / nnz and is the same
    for Bucket and FastRand."""
    w = make_workload(3, scale=0.01)
    deg = np.diff(w.rowptr).astype(np.int64)
    for W in (16, 32, 64, 128):
        _, cb = oracle.kept(w.rowptr, W, "bucket")
        _, cf = oracle.kept(w.rowptr, W, "fastrand")
        assert (cb == cf).all()
        assert int(cb.sum()) == int(np.minimum(deg, W).sum())
    _, cfull = oracle.kept(w.rowptr, 1, "full", stride=4)
    assert (cfull == deg).all()


def test_width_at_least_max_degree_is_full():
    w = make_workload(1)
    W = w.max_degree
    Yf, Df = oracle.spmm(w.rowptr, w.colidx, w.vals, w.X, w.F, 0, "full")
    pf, cf = oracle.kept(w.rowptr, 0, "full")
    for mode in ("bucket", "fastrand"):
        for seed in (0, 7):
            p, c = oracle.kept(w.rowptr, W, mode, seed)
            assert (c == cf).all() and (p == pf).all()
            Y, D = oracle.spmm(w.rowptr, w.colidx, w.vals, w.X, w.F, W, mode, seed)
            assert (Y == Yf).all() and (D == Df).all()


def test_determinism_and_seed_effect():
    w = make_workload(2, scale=0.02)
    W = 8
    a, _ = oracle.kept(w.rowptr, W, "fastrand", 5)
    b, _ = oracle.kept(w.rowptr, W, "fastrand", 5)
    assert (a == b).all()
    z, _ = oracle.kept(w.rowptr, W, "fastrand", 0)
    deg = np.diff(w.rowptr)
    assert (deg > W).any()
    changed = (a != z).any(axis=1)
    assert changed.any()
    assert not changed[deg <= W].any()          # rows that fit never move
    b0, _ = oracle.kept(w.rowptr, W, "bucket", 0)
    b5, _ = oracle.kept(w.rowptr, W, "bucket", 5)
    assert (b0 == b5).all()                     # Bucket ignores the seed
    # a subset of rows gives the same lists as the whole graph
    rows = np.array([3, 0, 17, w.N - 1])
    sub, _ = oracle.kept(w.rowptr, W, "fastrand", 5, rows=rows)
    assert (sub == a[rows]).all()


# --------------------------------------------------------------------------
# products
# --------------------------------------------------------------------------
def _dense_from_kept(w_rowptr, colidx, vals, pos, cnt, n):
    A = np.zeros((n, n), dtype=np.float64)
    for r in range(n):
        for p in pos[r, :cnt[r]]:
            A[r, colidx[p]] += np.float64(vals[p])
    return A


@pytest.mark.parametrize("F", [1, 3, 16, 41])
def test_full_mode_vs_dense_bruteforce(F):
    n = 48
    rowptr, colidx = random_csr(n, 5.0, seed=F, empty_frac=0.15)
    rng = np.random.default_rng(100 + F)
    vals = rng.standard_normal(colidx.size).astype(np.float32)
    X = rng.standard_normal((n, F + 3)).astype(np.float32)     # ldx > F
    A = np.zeros((n, n))
    for r in range(n):
        for p in range(rowptr[r], rowptr[r + 1]):
            A[r, colidx[p]] = vals[p]
    Y, D = oracle.spmm(rowptr, colidx, vals, X, F, 0, "full")
    Xd = X[:, :F].astype(np.float64)
    np.testing.assert_allclose(Y, A @ Xd, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(D, np.abs(A) @ np.abs(Xd), rtol=1e-13, atol=1e-13)
    empty = np.diff(rowptr) == 0
    assert empty.any() and (Y[empty] == 0).all() and (D[empty] == 0).all()


@pytest.mark.parametrize("mode", ["bucket", "fastrand"])
@pytest.mark.parametrize("W", [1, 2, 5, 64])
def test_sampled_product_vs_dense_of_kept_edges(mode, W):
    n = 40
    rowptr, colidx = random_csr(n, 7.0, seed=W)
    rng = np.random.default_rng(W)
    vals = rng.standard_normal(colidx.size).astype(np.float32)
    X = rng.uniform(-1, 1, (n, 5)).astype(np.float32)
    for seed in (0, 9):
        pos, cnt = oracle.kept(rowptr, W, mode, seed)
        deg = np.diff(rowptr)
        assert (cnt == np.minimum(deg, W)).all()
        for r in range(n):                       # distinct, inside the row
            p = pos[r, :cnt[r]]
            assert np.unique(p).size == cnt[r]
            assert ((p >= rowptr[r]) & (p < rowptr[r + 1])).all()
        A = _dense_from_kept(rowptr, colidx, vals, pos, cnt, n)
        Y, D = oracle.spmm(rowptr, colidx, vals, X, 5, W, mode, seed)
        Xd = X.astype(np.float64)
        np.testing.assert_allclose(Y, A @ Xd, rtol=1e-13, atol=1e-13)
        np.testing.assert_allclose(D, np.abs(A) @ np.abs(Xd), rtol=1e-13, atol=1e-13)


def test_full_mode_vs_scipy_csr_product():
    w = make_workload(2, scale=0.05)
    A = sp.csr_matrix((w.vals.astype(np.float64), w.colidx, w.rowptr), shape=(w.N, w.N))
    Xd = w.X.astype(np.float64)
    Y, D = oracle.spmm(w.rowptr, w.colidx, w.vals, w.X, w.F, 0, "full")
    np.testing.assert_allclose(Y, A @ Xd, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(D, abs(A) @ np.abs(Xd), rtol=1e-12, atol=1e-12)
    rows = np.array([5, 1, w.N - 1, 5])
    Ys, _ = oracle.spmm(w.rowptr, w.colidx, w.vals, w.X, w.F, 0, "full", rows=rows)
    assert (Ys == Y[rows]).all()


def test_bucket_product_vs_scipy_on_truncated_rows():
    """Bucket keeps each row's first W stored entries: the product must equal
    SciPy's on the matrix with every row cut to its first W entries."""
    w = make_workload(3, scale=0.005)
    W = 16
    deg = np.diff(w.rowptr)
    keep = np.concatenate([np.arange(w.rowptr[r], w.rowptr[r] + min(deg[r], W))
                           for r in range(w.N)])
    rp = np.zeros(w.N + 1, dtype=np.int64)
    rp[1:] = np.cumsum(np.minimum(deg, W))
    A = sp.csr_matrix((w.vals[keep].astype(np.float64), w.colidx[keep], rp), shape=(w.N, w.N))
    Y, _ = oracle.spmm(w.rowptr, w.colidx, w.vals, w.X, w.F, W, "bucket")
    np.testing.assert_allclose(Y, A @ w.X.astype(np.float64), rtol=1e-12, atol=1e-12)


def test_unweighted_graph_has_unit_values():
    rowptr, colidx = random_csr(64, 6.0, seed=2)
    X = np.random.default_rng(2).standard_normal((64, 4)).astype(np.float32)
    ones = np.ones(colidx.size, dtype=np.float32)
    for mode, W in (("full", 0), ("bucket", 3), ("fastrand", 3)):
        Y1, D1 = oracle.spmm(rowptr, colidx, None, X, 4, W, mode)
        Y2, D2 = oracle.spmm(rowptr, colidx, ones, X, 4, W, mode)
        assert (Y1 == Y2).all() and (D1 == D2).all()


def test_bad_arguments_are_rejected():
    rowptr, colidx = random_csr(16, 3.0, seed=1)
    X = np.zeros((16, 4), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.spmm(rowptr, colidx, None, X, 4, 0, "bucket")      # W < 1
    with pytest.raises(ValueError):
        oracle.spmm(rowptr, colidx, None, X, 4, 4, 7)             # unknown mode
    with pytest.raises(ValueError):
        oracle.spmm(rowptr, colidx, None, X, 4, 4, "bucket", rows=[16])
    with pytest.raises(ValueError):
        oracle.kept(rowptr, 0, "fastrand")


# --------------------------------------------------------------------------
# row normalisation (Section 6.1; this build's reading, see the oracle header)
# --------------------------------------------------------------------------
def test_row_factor_closed_forms():
    assert oracle.row_factor("none", 10, 4) == 1.0
    assert oracle.row_factor("mean", 10, 4) == 0.25
    assert oracle.row_factor("rsqrt", 10, 4) == 0.5
    assert oracle.row_factor("rescale", 10, 4) == 2.5
    assert oracle.row_factor("inv_degree", 10, 4) == 0.1
    for norm in ("mean", "rsqrt", "rescale", "inv_degree"):
        assert oracle.row_factor(norm, 0, 0) == 0.0
    assert oracle.row_factor("none", 0, 0) == 1.0


@pytest.mark.parametrize("norm", ["mean", "rsqrt", "rescale", "inv_degree"])
@pytest.mark.parametrize("mode,W", [("bucket", 3), ("fastrand", 3), ("full", 0), ("fastrand", 50)])
def test_normalised_product_vs_dense_bruteforce(norm, mode, W):
    n, F = 44, 6
    rowptr, colidx = random_csr(n, 7.0, seed=17, empty_frac=0.15)
    rng = np.random.default_rng(3)
    vals = rng.standard_normal(colidx.size).astype(np.float32)
    X = rng.standard_normal((n, F)).astype(np.float32)
    pos, cnt = oracle.kept(rowptr, W, mode, 4)
    A = _dense_from_kept(rowptr, colidx, vals, pos, cnt, n)
    deg = np.diff(rowptr).astype(np.float64)
    k = cnt.astype(np.float64)
    with np.errstate(divide="ignore", invalid="ignore"):
        f = {"mean": 1.0 / k, "rsqrt": 1.0 / np.sqrt(k), "rescale": deg / k, "inv_degree": 1.0 / deg}[norm]
    f = np.where(k > 0, f, 0.0)
    Y, D = oracle.spmm(rowptr, colidx, vals, X, F, W, mode, 4, norm=norm)
    Xd = X.astype(np.float64)
    np.testing.assert_allclose(Y, f[:, None] * (A @ Xd), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(D, f[:, None] * (np.abs(A) @ np.abs(Xd)), rtol=1e-13, atol=1e-13)


def test_normalisation_special_cases():
    w = make_workload(1)
    ones = np.ones((w.N, 3), dtype=np.float32)
    # mean of ones over any kept set is 1; rescale of unit values recovers the degree
    for mode, W in (("bucket", 4), ("fastrand", 4), ("full", 0)):
        Y, _ = oracle.spmm(w.rowptr, w.colidx, None, ones, 3, W, mode, 0, norm="mean")
        assert np.allclose(Y, 1.0, rtol=1e-15)
        Y, _ = oracle.spmm(w.rowptr, w.colidx, None, ones, 3, W, mode, 0, norm="rescale")
        assert np.allclose(Y, np.diff(w.rowptr)[:, None], rtol=1e-15)
    # unit values normalised by the original degree == the mean-aggregation values 1/d_i
    w3 = make_workload(3, scale=0.005)
    for mode, W in (("fastrand", 16), ("full", 0)):
        Ya, Da = oracle.spmm(w3.rowptr, w3.colidx, w3.vals, w3.X, w3.F, W, mode, 0)
        Yb, Db = oracle.spmm(w3.rowptr, w3.colidx, None, w3.X, w3.F, W, mode, 0, norm="inv_degree")
        np.testing.assert_allclose(Yb, Ya, rtol=1e-6, atol=1e-12)      # vals are 1/d rounded to fp32
    # nothing is dropped when W covers every row: rescale is the identity
    Yn, Dn = oracle.spmm(w.rowptr, w.colidx, w.vals, w.X, w.F, w.max_degree, "fastrand", 0)
    Yr, Dr = oracle.spmm(w.rowptr, w.colidx, w.vals, w.X, w.F, w.max_degree, "fastrand", 0, norm="rescale")
    assert (Yn == Yr).all() and (Dn == Dr).all()
    with pytest.raises(ValueError):
        oracle.spmm(w.rowptr, w.colidx, w.vals, w.X, w.F, 4, "bucket", 0, norm=9)


# --------------------------------------------------------------------------
# transposed product (backward pass of the sampled aggregation)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("norm", ["none", "mean", "rescale"])
@pytest.mark.parametrize("mode,W", [("bucket", 3), ("fastrand", 3), ("full", 0), ("fastrand", 50)])
def test_backward_vs_dense_transpose(mode, W, norm):
    n, F = 41, 5
    rowptr, colidx = random_csr(n, 7.0, seed=23, empty_frac=0.15)
    rng = np.random.default_rng(5)
    vals = rng.standard_normal(colidx.size).astype(np.float32)
    dY = rng.standard_normal((n, F + 2)).astype(np.float32)        # ldy > F
    pos, cnt = oracle.kept(rowptr, W, mode, 6)
    A = _dense_from_kept(rowptr, colidx, vals, pos, cnt, n)
    f = np.array([oracle.row_factor(norm, int(d), int(k)) for d, k in zip(np.diff(rowptr), cnt)])
    A = f[:, None] * A
    dX, D = oracle.spmm_backward(rowptr, colidx, vals, dY, F, W, mode, 6, norm=norm)
    dYd = dY[:, :F].astype(np.float64)
    np.testing.assert_allclose(dX, A.T @ dYd, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(D, np.abs(A).T @ np.abs(dYd), rtol=1e-13, atol=1e-13)


def test_backward_is_the_adjoint_of_forward():
    """<A_s X, dY> == <X, A_s^T dY> ties the backward oracle to the forward one."""
    w = make_workload(2, scale=0.03)
    rng = np.random.default_rng(9)
    dY = rng.standard_normal((w.N, w.F)).astype(np.float32)
    for mode, W, norm in (("fastrand", 8, "none"), ("bucket", 8, "mean"), ("full", 0, "rsqrt")):
        Y, _ = oracle.spmm(w.rowptr, w.colidx, w.vals, w.X, w.F, W, mode, 2, norm=norm)
        dX, _ = oracle.spmm_backward(w.rowptr, w.colidx, w.vals, dY, w.F, W, mode, 2, norm=norm)
        lhs = float((Y * dY.astype(np.float64)).sum())
        rhs = float((w.X.astype(np.float64) * dX).sum())
        assert abs(lhs - rhs) <= 1e-10 * max(1.0, abs(lhs))
    # full mode equals SciPy's transposed product
    A = sp.csr_matrix((w.vals.astype(np.float64), w.colidx, w.rowptr), shape=(w.N, w.N))
    dX, D = oracle.spmm_backward(w.rowptr, w.colidx, w.vals, dY, w.F, 0, "full")
    np.testing.assert_allclose(dX, A.T @ dY.astype(np.float64), rtol=1e-12, atol=1e-12)
