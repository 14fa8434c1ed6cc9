"""Pins of the RGMS oracle (CPU only): the dense definition through einsum, the special cases that reduce to
SpMM and to library products, the two-stage form of the same operator, and planted mistakes."""
import numpy as np
import scipy.sparse as sp

import oracle
import workloads


def tiny(seed=0, d_in=6, d_out=5):
    return workloads.make_hetero("hetero_tiny", seed=seed, d_in=d_in, d_out=d_out, scale=0.2)


def dense_tensor(w):
    A = np.zeros((w.n_rel, w.n, w.n))
    stacked = np.repeat(np.arange(w.n_rel * w.n), np.diff(w.indptr))
    A[stacked // w.n, stacked % w.n, w.indices] = w.values.astype(np.float64)
    return A


def slice_csr(w, r):
    lo, hi = w.indptr[r * w.n], w.indptr[(r + 1) * w.n]
    return (w.indptr[r * w.n:(r + 1) * w.n + 1] - lo).astype(np.int32), w.indices[lo:hi], w.values[lo:hi]


def test_rgms_matches_einsum_of_the_definition():
    for seed in range(4):
        w = tiny(seed)
        Y, S = oracle.rgms(w.n_rel, w.n, w.indptr, w.indices, w.values, w.X, w.W)
        A = dense_tensor(w)
        want = np.einsum("rij,jk,rkl->il", A, w.X.astype(np.float64), w.W.astype(np.float64))
        want_abs = np.einsum("rij,jk,rkl->il", np.abs(A), np.abs(w.X.astype(np.float64)), np.abs(w.W.astype(np.float64)))
        np.testing.assert_allclose(Y, want, rtol=0, atol=1e-12)
        np.testing.assert_allclose(S, want_abs, rtol=1e-12)
        assert Y.shape == (w.n, w.W.shape[2])
        empty = A.sum((0, 2)) == 0
        assert (Y[empty] == 0).all()


def test_rgms_single_relation_identity_weight_is_spmm():
    w = tiny(5, d_in=7, d_out=7)
    ip, ix, va = slice_csr(w, 2)
    eye = np.eye(7, dtype=np.float32)[None]
    Y = oracle.rgms(1, w.n, ip, ix, va, w.X, eye, want_abs=False)
    want = oracle.spmm_csr(w.n, ip, ix, va, w.X, want_abs=False)
    assert np.array_equal(Y, want)        # multiplying by exact 0 and 1 changes nothing


def test_rgms_shared_weight_factors_out():
    """W_r = W for every r  =>  Y = (sum_r A_r) X W, with library products."""
    w = tiny(6)
    Wsame = np.repeat(w.W[:1], w.n_rel, axis=0)
    Y = oracle.rgms(w.n_rel, w.n, w.indptr, w.indices, w.values, w.X, Wsame, want_abs=False)
    stacked = sp.csr_matrix((w.values.astype(np.float64), w.indices, w.indptr), shape=(w.n_rel * w.n, w.n))
    summed = sum(stacked[r * w.n:(r + 1) * w.n] for r in range(w.n_rel))
    want = (summed @ w.X.astype(np.float64)) @ w.W[0].astype(np.float64)
    np.testing.assert_allclose(Y, want, rtol=0, atol=1e-12)


def test_rgms_equals_its_two_stage_form():
    """T_r = X W_r, Y = sum_r A_r T_r (the two equations the paper gives for existing libraries); the second
    stage runs through the SpMM oracle.  T is rounded to float32 nowhere: fed as float64 via two float32 halves."""
    w = tiny(7)
    Y, S = oracle.rgms(w.n_rel, w.n, w.indptr, w.indices, w.values, w.X, w.W)
    want = np.zeros_like(Y)
    for r in range(w.n_rel):
        T = w.X.astype(np.float64) @ w.W[r].astype(np.float64)
        hi = T.astype(np.float32)
        lo = (T - hi.astype(np.float64)).astype(np.float32)
        ip, ix, va = slice_csr(w, r)
        want += oracle.spmm_csr(w.n, ip, ix, va, hi, want_abs=False) + oracle.spmm_csr(w.n, ip, ix, va, lo, want_abs=False)
    assert (np.abs(Y - want) <= 1e-12 * np.maximum(S, 1e-300)).all()


def test_rgms_scales_exactly():
    w = tiny(8)
    Y = oracle.rgms(w.n_rel, w.n, w.indptr, w.indices, w.values, w.X, w.W, want_abs=False)
    Y2 = oracle.rgms(w.n_rel, w.n, w.indptr, w.indices, 2 * w.values, 4 * w.X, 0.5 * w.W, want_abs=False)
    assert np.array_equal(Y2, 4 * Y)       # powers of two: exact


def test_checks_catch_planted_rgms_mistakes():
    w = tiny(9, d_in=5, d_out=5)       # square weights, so a transposed W is at least multipliable
    A = dense_tensor(w)
    X, W = w.X.astype(np.float64), w.W.astype(np.float64)
    want = np.einsum("rij,jk,rkl->il", A, X, W)
    wrong = {
        "W transposed": np.einsum("rij,jk,rlk->il", A, X, W),
        "weights of the next relation": np.einsum("rij,jk,rkl->il", A, X, np.roll(W, 1, axis=0)),
        "A transposed": np.einsum("rji,jk,rkl->il", A, X, W),
        "last relation missing": np.einsum("rij,jk,rkl->il", A[:-1], X, W[:-1]),
        "relations summed before the weights": np.einsum("ij,jk,kl->il", A.sum(0), X, W.mean(0)),
    }
    for name, Y in wrong.items():
        assert not np.allclose(Y, want, rtol=1e-9, atol=1e-12), name


def test_hetero_generator_shapes():
    w = workloads.make_hetero("hetero_a")
    assert w.indptr.shape == (w.n_rel * w.n + 1,) and w.indptr[-1] == w.nnz and w.n == 7262 and w.n_rel == 45
    assert abs(w.nnz - 48810) < 0.01 * 48810
    rows = np.repeat(np.arange(w.n_rel * w.n), np.diff(w.indptr))
    key = rows.astype(np.int64) * w.n + w.indices
    assert (np.diff(key) > 0).all()                       # strictly ascending inside and across stacked rows
    counts = np.diff(w.indptr)
    np.testing.assert_allclose(w.values, (1.0 / counts[rows]).astype(np.float32))
