"""Pins of the CPU oracle to things other than itself (no GPU needed).

SpMM half: brute-force dense products on tiny matrices, A = I, X = ones
(row sums / degrees), linearity, and SciPy's CSR product as an independent
textbook routine.  Format half: the hand-worked hyb(2,2) example, the
properties Section 4.2.1 fixes (tests/hyb_checks.py), the bucket count of the
hyb(2,2) figure, special cases, exhaustive small 0/1 matrices, and planted
mistakes that the checks must catch.
"""
import copy
import itertools
import os

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
import workloads
from hyb_checks import assert_same_hyb, decode_and_check, load_golden

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hyb_2_2_example.txt")


def dense_of(n_rows, n_cols, indptr, indices, values):
    A = np.zeros((n_rows, n_cols), dtype=np.float64)
    for r in range(n_rows):
        for q in range(indptr[r], indptr[r + 1]):
            A[r, indices[q]] = np.float64(values[q])
    return A


def small_workload(seed, n_rows=37, n_cols=53, feat=7, max_deg=20, empty_frac=0.2):
    rng = np.random.default_rng(seed)
    deg = rng.integers(1, max_deg + 1, n_rows)
    deg[rng.random(n_rows) < empty_frac] = 0
    return workloads.random_csr(n_rows, n_cols, np.minimum(deg, n_cols), seed, feat)


# ----------------------------------------------------------------- SpMM half

@pytest.mark.parametrize("seed", range(6))
def test_spmm_matches_dense_brute_force(seed):
    w = small_workload(seed)
    A = dense_of(w.n_rows, w.n_cols, w.indptr, w.indices, w.values)
    Y, S = oracle.spmm_csr(w.n_rows, w.indptr, w.indices, w.values, w.X)
    want = np.zeros((w.n_rows, w.feat))
    want_abs = np.zeros((w.n_rows, w.feat))
    Xd = w.X.astype(np.float64)
    for i in range(w.n_rows):           # the definition, term by term
        for j in range(w.n_cols):
            if A[i, j] != 0.0:
                want[i] += A[i, j] * Xd[j]
                want_abs[i] += np.abs(A[i, j] * Xd[j])
    np.testing.assert_allclose(Y, want, rtol=0, atol=1e-13)
    np.testing.assert_allclose(S, want_abs, rtol=1e-14, atol=0)
    empty = np.diff(w.indptr) == 0
    assert empty.any() and (Y[empty] == 0.0).all()


def test_spmm_identity_returns_x_exactly():
    n, feat = 41, 9
    rng = np.random.default_rng(3)
    X = rng.standard_normal((n, feat)).astype(np.float32)
    indptr = np.arange(n + 1, dtype=np.int32)
    indices = np.arange(n, dtype=np.int32)
    Y, S = oracle.spmm_csr(n, indptr, indices, np.ones(n, np.float32), X)
    assert np.array_equal(Y, X.astype(np.float64))
    assert np.array_equal(S, np.abs(X.astype(np.float64)))


def test_spmm_ones_gives_row_sums_and_degrees():
    w = small_workload(11, feat=3)
    X = np.ones((w.n_cols, 3), np.float32)
    Y = oracle.spmm_csr(w.n_rows, w.indptr, w.indices, w.values, X, want_abs=False)
    rowsum = np.array([np.sum(w.values[w.indptr[r]:w.indptr[r + 1]].astype(np.float64))
                       for r in range(w.n_rows)])
    np.testing.assert_allclose(Y, np.repeat(rowsum[:, None], 3, 1), rtol=0, atol=1e-13)
    Yd = oracle.spmm_csr(w.n_rows, w.indptr, w.indices, np.ones_like(w.values), X, want_abs=False)
    assert np.array_equal(Yd, np.repeat(np.diff(w.indptr)[:, None], 3, 1).astype(np.float64))


def test_spmm_is_linear_in_x():
    w = small_workload(5)
    rng = np.random.default_rng(9)
    # dyadic inputs keep every fp64 operation exact, so linearity holds bit for bit
    X1 = rng.integers(-8, 9, w.X.shape).astype(np.float32)
    X2 = rng.integers(-8, 9, w.X.shape).astype(np.float32)
    vals = rng.integers(-4, 5, w.values.shape).astype(np.float32)
    f = lambda X: oracle.spmm_csr(w.n_rows, w.indptr, w.indices, vals, X, want_abs=False)
    assert np.array_equal(f(2 * X1 + X2), 2 * f(X1) + f(X2))


@pytest.mark.parametrize("name", ["tiny", "small"])
def test_spmm_matches_scipy_csr(name):
    w = workloads.make_config(name)
    A = sp.csr_matrix((w.values.astype(np.float64), w.indices, w.indptr), shape=(w.n_rows, w.n_cols))
    want = A @ w.X.astype(np.float64)
    Y, S = oracle.spmm_csr(w.n_rows, w.indptr, w.indices, w.values, w.X)
    err = np.abs(Y - want)
    assert (err <= 1e-13 * np.maximum(S, 1e-300)).all()


def test_spmm_rows_subset_equals_full():
    w = workloads.make_config("tiny")
    Y, S = oracle.spmm_csr(w.n_rows, w.indptr, w.indices, w.values, w.X)
    rows = np.array([0, 5, 17, w.n_rows - 1, 5], dtype=np.int32)
    Yr, Sr = oracle.spmm_csr_rows(rows, w.indptr, w.indices, w.values, w.X)
    assert np.array_equal(Yr, Y[rows]) and np.array_equal(Sr, S[rows])


# --------------------------------------------------------------- format half

def test_hyb_hand_worked_example():
    g = load_golden(GOLDEN)
    ints = lambda k: np.array(g[k], dtype=np.int64)
    n_rows, n_cols, c, k = (int(g[x][0]) for x in ("n_rows", "n_cols", "c", "k"))
    h = oracle.hyb_build(n_rows, n_cols, ints("indptr"), ints("indices"),
                         np.array(g["values"], np.float32), c, k)
    for name in h.ARRAY_NAMES:
        got = getattr(h, name)
        want = np.array(g[name], dtype=got.dtype)
        assert np.array_equal(got, want), name
    # hyb(2,2): six ELL sub-matrices, three per partition (figure of Section 4.2.1)
    assert h.bucket_row_ptr.shape[0] - 1 == 6
    X = np.ones((n_cols, 1), np.float32)
    assert np.array_equal(oracle.spmm_hyb(h, X).ravel(), np.array(g["y_ones"], np.float64))
    assert np.array_equal(
        oracle.spmm_csr(n_rows, ints("indptr"), ints("indices"), np.array(g["values"], np.float32),
                        X, want_abs=False).ravel(), np.array(g["y_ones"], np.float64))


@pytest.mark.parametrize("seed,c,k", [(0, 1, 0), (1, 1, 3), (2, 2, 2), (3, 3, 1), (4, 5, 4),
                                      (5, 7, 0), (6, 16, 2), (7, 60, 3), (8, 4, 30)])
def test_hyb_properties_and_reconstruction(seed, c, k):
    w = small_workload(seed, n_rows=45, n_cols=57, max_deg=40)
    h = oracle.hyb_build(w.n_rows, w.n_cols, w.indptr, w.indices, w.values, c, k)
    stats = decode_and_check(h, w.n_rows, w.n_cols, w.indptr, w.indices, w.values)
    assert stats["pads"] < max(1, stats["nnz"])          # pads < half of each padded row
    # the two halves agree: SpMM from the hyb arrays == SpMM by definition
    Y, S = oracle.spmm_csr(w.n_rows, w.indptr, w.indices, w.values, w.X)
    Yh = oracle.spmm_hyb(h, w.X)
    assert (np.abs(Y - Yh) <= 1e-12 * np.maximum(S, 1e-300)).all()


def test_hyb_special_cases():
    w = small_workload(21, n_rows=30, n_cols=64, max_deg=33)
    deg = np.diff(w.indptr)
    # one partition, k large: nothing in the remainder, each row in bucket ceil(log2 deg)
    h = oracle.hyb_build(w.n_rows, w.n_cols, w.indptr, w.indices, w.values, 1, 6)
    assert h.rem_row.size == 0 and h.rem_col.size == 0
    for i in range(7):
        rows = h.ell_row[h.bucket_row_ptr[i]:h.bucket_row_ptr[i + 1]]
        want = np.flatnonzero((deg > (1 << i) // 2) & (deg <= (1 << i)) & (deg > 0)) if i else np.flatnonzero(deg == 1)
        assert np.array_equal(rows, want)
    # k = 0: only single-entry pieces are ELL, everything else is remainder
    h0 = oracle.hyb_build(w.n_rows, w.n_cols, w.indptr, w.indices, w.values, 1, 0)
    assert np.array_equal(h0.ell_row, np.flatnonzero(deg == 1))
    assert np.array_equal(h0.rem_row, np.flatnonzero(deg > 1))
    assert h0.rem_col.size == deg[deg > 1].sum()
    # more partitions than columns: w = 1, every piece has length 1
    hc = oracle.hyb_build(w.n_rows, w.n_cols, w.indptr, w.indices, w.values, 100, 2)
    assert hc.w == 1 and hc.ell_col.size == w.nnz and hc.rem_col.size == 0
    decode_and_check(hc, w.n_rows, w.n_cols, w.indptr, w.indices, w.values)
    # empty matrix
    he = oracle.hyb_build(3, 5, np.zeros(4, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32), 2, 2)
    assert he.ell_row.size == 0 and he.bucket_row_ptr.tolist() == [0] * 7 and he.rem_ptr.tolist() == [0]


def test_hyb_exhaustive_small_binary_matrices():
    n_rows, n_cols = 3, 4
    for pattern in itertools.product([0, 1], repeat=n_rows * n_cols):
        M = np.array(pattern).reshape(n_rows, n_cols)
        indptr = np.concatenate([[0], np.cumsum(M.sum(1))]).astype(np.int32)
        indices = np.concatenate([np.flatnonzero(M[r]) for r in range(n_rows)]).astype(np.int32)
        values = (np.arange(indices.size) + 1).astype(np.float32)
        for c, k in ((1, 0), (1, 1), (2, 1), (2, 0), (3, 2)):
            h = oracle.hyb_build(n_rows, n_cols, indptr, indices, values, c, k)
            decode_and_check(h, n_rows, n_cols, indptr, indices, values)


def test_hyb_rejects_bad_input():
    with pytest.raises(ValueError):
        oracle.hyb_build(1, 4, [0, 2], [2, 1], [1.0, 1.0], 1, 1)      # descending
    with pytest.raises(ValueError):
        oracle.hyb_build(1, 4, [0, 2], [1, 1], [1.0, 1.0], 1, 1)      # duplicate
    with pytest.raises(ValueError):
        oracle.hyb_build(1, 4, [0, 1], [4], [1.0], 1, 1)              # out of range
    with pytest.raises(ValueError):
        oracle.hyb_build(1, 4, [0, 1], [0], [1.0], 0, 1)              # c < 1


@pytest.mark.parametrize("name", ["tiny", "small"])
def test_hyb_on_named_configs(name):
    w = workloads.make_config(name)
    h = oracle.hyb_build(w.n_rows, w.n_cols, w.indptr, w.indices, w.values, w.n_col_parts, w.max_bucket_log2)
    stats = decode_and_check(h, w.n_rows, w.n_cols, w.indptr, w.indices, w.values)
    assert stats["pads"] < stats["nnz"]


def _mutations(h):
    """Plausible construction mistakes, planted in the oracle's output."""
    m = copy.deepcopy(h); m.ell_row[[0, 1]] = m.ell_row[[1, 0]]; yield "rows swapped", m
    m = copy.deepcopy(h); m.ell_col[0], m.ell_col[1] = h.ell_col[1], h.ell_col[0]; yield "cols swapped", m
    m = copy.deepcopy(h)
    pad = np.flatnonzero(h.ell_val.view(np.uint32) == 0)
    m.ell_val[pad[0]] = -0.0; yield "pad is -0.0", m
    m = copy.deepcopy(h); m.ell_col[pad[0]] += 1; yield "pad column not repeated", m
    m = copy.deepcopy(h); m.ell_val[2] = np.float32(m.ell_val[2]) * np.float32(1.0000001); yield "value changed", m
    m = copy.deepcopy(h); m.rem_row[0] += 1; yield "remainder row shifted", m


def test_checks_catch_planted_mistakes():
    w = small_workload(2, n_rows=45, n_cols=57, max_deg=40)
    h = oracle.hyb_build(w.n_rows, w.n_cols, w.indptr, w.indices, w.values, 2, 2)
    decode_and_check(h, w.n_rows, w.n_cols, w.indptr, w.indices, w.values)
    assert h.rem_row.size > 0
    for what, m in _mutations(h):
        with pytest.raises(AssertionError):
            decode_and_check(m, w.n_rows, w.n_cols, w.indptr, w.indices, w.values)
            pytest.fail(f"not caught: {what}")
        with pytest.raises(AssertionError):
            assert_same_hyb(m, h)
