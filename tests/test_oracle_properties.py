"""Property tests of the CPU oracle (hypothesis): invariants the paper and the
mathematics fix for any input -- kept counts (Section 4.2), distinct in-row
picks, linearity of the product in X, |Y| <= sum |a||x|, row sums for X = 1."""
import numpy as np
from hypothesis import given, settings, strategies as st

import oracle
from workloads import random_csr

MODES = ("bucket", "fastrand")


@settings(max_examples=300, deadline=None)
@given(n=st.integers(1, 200_000), W=st.integers(1, 4096), seed=st.integers(0, 2 ** 64 - 1),
       row=st.integers(0, 10 ** 6), mode=st.sampled_from(MODES))
def test_kept_slots_are_distinct_positions_of_the_row(n, W, seed, row, mode):
    k = oracle.kept_count(mode, n, W)
    assert k == min(n, W)
    step = max(1, k // 64)                      # sample the slots of long lists
    idx = [oracle.sample_index(mode, seed, row, i, n, W) for i in range(0, k, step)]
    assert all(0 <= v < n for v in idx)
    assert len(set(idx)) == len(idx)
    if n <= W or mode == "bucket":
        assert idx == list(range(0, k, step))


@settings(max_examples=60, deadline=None)
@given(n=st.integers(2, 3000), frac=st.floats(0.01, 0.99), seed=st.integers(0, 2 ** 32))
def test_all_slots_distinct_for_any_width_below_n(n, frac, seed):
    W = max(1, min(n - 1, int(n * frac)))
    pos, cnt = oracle.kept(np.array([0, n], dtype=np.int32), W, "fastrand", seed)
    assert cnt[0] == W and np.unique(pos[0]).size == W
    assert pos[0].min() >= 0 and pos[0].max() < n


@settings(max_examples=25, deadline=None)
@given(gseed=st.integers(0, 10_000), W=st.integers(1, 12), seed=st.integers(0, 99),
       mode=st.sampled_from(MODES + ("full",)))
def test_product_is_linear_in_X_and_bounded_by_denominator(gseed, W, seed, mode):
    n, F = 60, 7
    rowptr, colidx = random_csr(n, 6.0, seed=gseed, empty_frac=0.1)
    rng = np.random.default_rng(gseed)
    vals = rng.standard_normal(colidx.size).astype(np.float32)
    X1 = rng.standard_normal((n, F)).astype(np.float32)
    X2 = rng.standard_normal((n, F)).astype(np.float32)
    Y1, D1 = oracle.spmm(rowptr, colidx, vals, X1, F, W, mode, seed)
    Y2, D2 = oracle.spmm(rowptr, colidx, vals, X2, F, W, mode, seed)
    Xs = (X1.astype(np.float64) * 2 - X2.astype(np.float64) * 3)
    # the combination is formed in float64 and rounded once, so compare loosely
    Ys, _ = oracle.spmm(rowptr, colidx, vals, Xs.astype(np.float32), F, W, mode, seed)
    scale = 2 * D1 + 3 * D2
    assert (np.abs(Ys - (2 * Y1 - 3 * Y2)) <= 1e-6 * scale + 1e-12).all()
    assert (np.abs(Y1) <= D1 * (1 + 1e-12) + 1e-300).all()


@settings(max_examples=25, deadline=None)
@given(gseed=st.integers(0, 10_000), W=st.integers(1, 20), seed=st.integers(0, 99),
       mode=st.sampled_from(MODES))
def test_unit_inputs_count_the_kept_entries(gseed, W, seed, mode):
    n = 80
    rowptr, colidx = random_csr(n, 8.0, seed=gseed, empty_frac=0.1)
    X = np.ones((n, 2), dtype=np.float32)
    Y, D = oracle.spmm(rowptr, colidx, None, X, 2, W, mode, seed)
    k = np.minimum(np.diff(rowptr), W).astype(np.float64)
    assert (Y == k[:, None]).all() and (D == k[:, None]).all()
    Yf, _ = oracle.spmm(rowptr, colidx, None, X, 2, 0, "full", seed)
    assert (Yf == np.diff(rowptr)[:, None]).all()
