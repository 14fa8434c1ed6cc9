"""Pins of the SDDMM oracle (CPU only): the dense definition through a library
matrix product, closed forms, the identity that ties it to the SpMM oracle,
and planted mistakes that these checks must catch."""
import numpy as np
import pytest

import oracle
import workloads


def small_workload(seed, n_rows=29, n_cols=41, feat=9, max_deg=17, empty_frac=0.2):
    rng = np.random.default_rng(seed)
    deg = rng.integers(1, max_deg + 1, n_rows)
    deg[rng.random(n_rows) < empty_frac] = 0
    w = workloads.random_csr(n_rows, n_cols, np.minimum(deg, n_cols), seed, feat)
    Xr = rng.standard_normal((n_rows, feat)).astype(np.float32)    # the left operand has one row per row of A
    return w, Xr


def rows_of(indptr):
    return np.repeat(np.arange(len(indptr) - 1), np.diff(indptr))


def dense_sddmm(w, Xr, Yt):
    """A .* (X Y) with a dense fp64 matrix product (Y = Yt^T is d x n_cols), read back at the stored positions."""
    P = Xr.astype(np.float64) @ Yt.astype(np.float64).T
    r = rows_of(w.indptr)
    return w.values.astype(np.float64) * P[r, w.indices]


@pytest.mark.parametrize("seed", range(5))
def test_sddmm_matches_dense_product(seed):
    w, Xr = small_workload(seed)            # 29 x 41: a transposed operand cannot even be indexed the same way
    B, M = oracle.sddmm_csr(w.n_rows, w.indptr, w.indices, w.values, Xr, w.X)
    np.testing.assert_allclose(B, dense_sddmm(w, Xr, w.X), rtol=1e-13, atol=1e-14)
    assert B.shape == (w.nnz,) and (M >= np.abs(B) * (1 - 1e-12)).all()
    absP = np.abs(Xr.astype(np.float64)) @ np.abs(w.X.astype(np.float64)).T
    np.testing.assert_allclose(M, np.abs(w.values.astype(np.float64)) * absP[rows_of(w.indptr), w.indices], rtol=1e-13)


def test_sddmm_closed_forms():
    w, _ = small_workload(11, feat=16)
    ones_r = np.ones((w.n_rows, 16), np.float32)
    ones_c = np.ones((w.n_cols, 16), np.float32)
    B = oracle.sddmm_csr(w.n_rows, w.indptr, w.indices, w.values, ones_r, ones_c, want_abs=False)
    assert np.array_equal(B, 16.0 * w.values.astype(np.float64))          # X = Y = 1: d * A_ij exactly
    # one-hot features: B_ij = A_ij when row i and column j carry the same label, else 0
    rng = np.random.default_rng(3)
    lab_r, lab_c = rng.integers(0, 16, w.n_rows), rng.integers(0, 16, w.n_cols)
    Xr = np.eye(16, dtype=np.float32)[lab_r]
    Yt = np.eye(16, dtype=np.float32)[lab_c]
    B = oracle.sddmm_csr(w.n_rows, w.indptr, w.indices, w.values, Xr, Yt, want_abs=False)
    same = lab_r[rows_of(w.indptr)] == lab_c[w.indices]
    assert same.any() and (~same).any()
    assert np.array_equal(B, np.where(same, w.values.astype(np.float64), 0.0))


def test_sddmm_scales_exactly_with_a_and_x():
    w, Xr = small_workload(5)
    B = oracle.sddmm_csr(w.n_rows, w.indptr, w.indices, w.values, Xr, w.X, want_abs=False)
    B2 = oracle.sddmm_csr(w.n_rows, w.indptr, w.indices, 2.0 * w.values, 4.0 * Xr, w.X, want_abs=False)
    assert np.array_equal(B2, 8.0 * B)       # powers of two: exact


@pytest.mark.parametrize("seed", range(3))
def test_sddmm_row_sums_tie_to_spmm_oracle(seed):
    """sum_j B_ij = X[i,:] . (A Yt)[i,:]: the right-hand side comes from the SpMM oracle."""
    w, Xr = small_workload(20 + seed)
    B = oracle.sddmm_csr(w.n_rows, w.indptr, w.indices, w.values, Xr, w.X, want_abs=False)
    AY, S = oracle.spmm_csr(w.n_rows, w.indptr, w.indices, w.values, w.X)
    want = (Xr.astype(np.float64) * AY).sum(1)
    got = np.zeros(w.n_rows)
    np.add.at(got, rows_of(w.indptr), B)
    scale = (np.abs(Xr.astype(np.float64)) * S).sum(1) + 1e-300
    assert (np.abs(got - want) / scale).max() < 1e-13


def test_sddmm_named_config_against_dense():
    w = workloads.make_config("tiny")
    rng = np.random.default_rng(0)
    Xr = rng.standard_normal((w.n_rows, w.feat)).astype(np.float32)
    B = oracle.sddmm_csr(w.n_rows, w.indptr, w.indices, w.values, Xr, w.X, want_abs=False)
    np.testing.assert_allclose(B, dense_sddmm(w, Xr, w.X), rtol=1e-12, atol=1e-14)


def test_checks_catch_planted_sddmm_mistakes():
    """Plausible mistakes (dropped factor, swapped operands, wrong column, a short sum) each break a pin above."""
    w, Xr = small_workload(2, n_rows=33, n_cols=33)     # square, so that swapped operands are at least indexable
    want = dense_sddmm(w, Xr, w.X)
    r = rows_of(w.indptr)
    X64, Y64, a = Xr.astype(np.float64), w.X.astype(np.float64), w.values.astype(np.float64)
    wrong = {
        "A dropped": (X64[r] * Y64[w.indices]).sum(1),
        "operands swapped": a * (X64[w.indices] * Y64[r]).sum(1),
        "row used for the column": a * (X64[r] * Y64[r]).sum(1),
        "last k missing": a * (X64[r, :-1] * Y64[w.indices, :-1]).sum(1),
        "values shifted by one": np.roll(a, 1) * (X64[r] * Y64[w.indices]).sum(1),
    }
    for name, B in wrong.items():
        assert not np.allclose(B, want, rtol=1e-9, atol=1e-12), name
