"""Robustness of the test infrastructure itself.

1. The C oracles and the C column sampler are rebuilt as a stand-alone program with AddressSanitizer and
   UndefinedBehaviorSanitizer (host code only) and run on the inputs of the pins: ragged shapes, empty rows and
   partitions, rows longer than every bucket, the golden example, invalid inputs.  The sanitized program must finish
   without a report and return what the ordinary shared-library build returns.  An out-of-bounds read that happens
   to land on mapped memory would pass every value pin; this is the test that sees it.
2. A property test (hypothesis) over random CSR matrices and random (c, k): the arrays the format oracle builds
   pass every structural check of Section 4.2.1 and SpMM evaluated from them equals SpMM by definition.
"""
import os
import shutil
import subprocess

import numpy as np
import pytest
from hypothesis import HealthCheck, given, settings, strategies as st

import oracle
import workloads
from hyb_checks import ARRAY_NAMES, decode_and_check, load_golden

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SOURCES = [os.path.join(HERE, "sanitized_oracle_main.c"), os.path.join(ROOT, "oracle", "sddmm_oracle.c"),
           os.path.join(ROOT, "oracle", "rgms_oracle.c"), os.path.join(ROOT, "workloads", "colsample.c")]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:halt_on_error=1",
           UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1", OMP_NUM_THREADS="3")


@pytest.fixture(scope="module")
def prog(tmp_path_factory):
    """The sanitized program.  The sanitizer runtimes are linked statically, so nothing has to be preloaded."""
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    exe = str(tmp_path_factory.mktemp("sanitized") / "oracle_sanitized")
    subprocess.check_call(["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           "-static-libasan", "-static-libubsan", "-o", exe, *SOURCES, "-lm"])
    return exe


def run(prog, mode, header, arrays, tmp_path):
    fin, fout = str(tmp_path / "in.bin"), str(tmp_path / "out.bin")
    with open(fin, "wb") as f:
        np.asarray(header, dtype=np.int64).tofile(f)
        for a in arrays:
            np.ascontiguousarray(a).tofile(f)
    p = subprocess.run([prog, mode, fin, fout], env=ENV, capture_output=True, text=True, timeout=300)
    assert p.returncode == 0, f"sanitized {mode} run failed ({p.returncode}):\n{p.stderr[-4000:]}"
    assert "runtime error" not in p.stderr and "AddressSanitizer" not in p.stderr, p.stderr[-4000:]
    return np.fromfile(fout, dtype=np.uint8)


class Reader:
    def __init__(self, raw):
        self.raw, self.at = raw, 0

    def take(self, n, dtype):
        size = n * np.dtype(dtype).itemsize
        out = self.raw[self.at:self.at + size].view(dtype)
        assert out.shape[0] == n, "the sanitized program wrote less than expected"
        self.at += size
        return out

    def done(self):
        return self.at == self.raw.shape[0]


def hyb_case(prog, tmp_path, n_rows, n_cols, indptr, indices, values, X, c, k, seed=0):
    """Runs one input through the sanitized program and compares everything with the shared-library oracle."""
    feat = X.shape[1]
    X2 = np.random.default_rng(seed).standard_normal((n_rows, feat)).astype(np.float32)
    raw = run(prog, "hyb", [n_rows, n_cols, indices.shape[0], feat, c, k],
              [indptr.astype(np.int32), indices.astype(np.int32), values.astype(np.float32), X, X2], tmp_path)
    rd = Reader(raw)
    rc = int(rd.take(1, np.int64)[0])
    try:
        want = oracle.hyb_build(n_rows, n_cols, indptr, indices, values, c, k)
    except ValueError:
        assert rc != 0 and rd.done()
        return rc
    assert rc == 0
    B, R, S, M, T = (int(v) for v in rd.take(5, np.int64))
    sizes = dict(bucket_row_ptr=(B + 1, np.int64), bucket_slot_ptr=(B + 1, np.int64), ell_row=(R, np.int32),
                 ell_col=(S, np.int32), ell_val=(S, np.float32), rem_part_ptr=(c + 1, np.int32),
                 rem_row=(M, np.int32), rem_ptr=(M + 1, np.int64), rem_col=(T, np.int32), rem_val=(T, np.float32))
    for name in ARRAY_NAMES:
        got = rd.take(*sizes[name])
        ref = getattr(want, name)
        assert got.shape == ref.shape and got.tobytes() == ref.tobytes(), name
    ny = n_rows * feat
    Y, Sabs = oracle.spmm_csr(n_rows, indptr, indices, values, X)
    assert np.array_equal(rd.take(ny, np.float64), Y.ravel())
    assert np.array_equal(rd.take(ny, np.float64), Sabs.ravel())
    assert np.array_equal(rd.take(ny, np.float64), oracle.spmm_hyb(want, X).ravel())
    sel = np.arange(0, n_rows, 2, dtype=np.int32)
    assert np.array_equal(rd.take(sel.shape[0] * feat, np.float64), Y[sel].ravel())
    Bv, Mv = oracle.sddmm_csr(n_rows, indptr, indices, values, X2, X)
    assert np.array_equal(rd.take(indices.shape[0], np.float64), Bv)
    assert np.array_equal(rd.take(indices.shape[0], np.float64), Mv)
    assert rd.done()
    return 0


@pytest.mark.parametrize("seed,n_rows,n_cols,c,k,max_deg", [
    (0, 37, 53, 1, 0, 20), (1, 37, 53, 3, 2, 20), (2, 64, 64, 4, 5, 64), (3, 1, 1, 1, 0, 1), (4, 200, 17, 5, 1, 17),
    (5, 90, 1000, 7, 3, 300), (6, 33, 8, 8, 6, 8), (7, 50, 20, 20, 0, 20), (8, 300, 301, 2, 10, 301)])
def test_sanitized_hyb_spmm_sddmm(prog, tmp_path, seed, n_rows, n_cols, c, k, max_deg):
    rng = np.random.default_rng(seed)
    deg = np.minimum(rng.integers(0, max_deg + 1, n_rows), n_cols)
    deg[rng.random(n_rows) < 0.2] = 0
    deg[rng.integers(0, n_rows)] = min(max_deg, n_cols)
    w = workloads.random_csr(n_rows, n_cols, deg, seed, 5)
    assert hyb_case(prog, tmp_path, n_rows, n_cols, w.indptr, w.indices, w.values, w.X, c, k, seed) == 0


def test_sanitized_golden_example(prog, tmp_path):
    g = load_golden(os.path.join(HERE, "golden", "hyb_2_2_example.txt"))
    n_rows, n_cols = int(g["n_rows"][0]), int(g["n_cols"][0])
    indptr = np.array(g["indptr"], dtype=np.int32)
    indices = np.array(g["indices"], dtype=np.int32)
    values = np.array(g["values"], dtype=np.float32)
    X = np.arange(n_cols * 3, dtype=np.float32).reshape(n_cols, 3)
    assert hyb_case(prog, tmp_path, n_rows, n_cols, indptr, indices, values, X, int(g["c"][0]), int(g["k"][0])) == 0


def test_sanitized_named_config_and_empty_matrix(prog, tmp_path):
    w = workloads.make_config("tiny")
    X = w.X[:, :4].copy()
    assert hyb_case(prog, tmp_path, w.n_rows, w.n_cols, w.indptr, w.indices, w.values, X, w.n_col_parts, w.max_bucket_log2) == 0
    z = np.zeros(0, dtype=np.int32)
    assert hyb_case(prog, tmp_path, 6, 9, np.zeros(7, dtype=np.int32), z, z.astype(np.float32),
                    np.ones((9, 2), dtype=np.float32), 2, 3) == 0


def test_sanitized_invalid_input_is_refused_without_a_stray_read(prog, tmp_path):
    X = np.ones((5, 2), dtype=np.float32)
    ip = np.array([0, 2, 3], dtype=np.int32)
    va = np.ones(3, dtype=np.float32)
    for indices in ([3, 1, 0], [1, 1, 0], [0, 5, 2], [-1, 2, 2]):     # descending, repeated, too large, negative
        assert hyb_case(prog, tmp_path, 2, 5, ip, np.array(indices, dtype=np.int32), va, X, 2, 2) != 0
    good = np.array([0, 4, 2], dtype=np.int32)
    assert hyb_case(prog, tmp_path, 2, 5, ip, good, va, X, 0, 2) != 0           # c < 1
    assert hyb_case(prog, tmp_path, 2, 5, ip, good, va, X, 2, -1) != 0          # k < 0
    assert hyb_case(prog, tmp_path, 2, 5, np.array([0, 3, 2], dtype=np.int32), good, va, X, 2, 2) != 0   # indptr falls


def test_sanitized_rgms(prog, tmp_path):
    for seed, d_in, d_out in ((0, 8, 5), (1, 3, 16)):
        w = workloads.make_hetero("hetero_tiny", seed=seed, d_in=d_in, d_out=d_out)
        raw = run(prog, "rgms", [w.n_rel, w.n, w.nnz, d_in, d_out, 0], [w.indptr, w.indices, w.values, w.X, w.W], tmp_path)
        rd = Reader(raw)
        Y, S = oracle.rgms(w.n_rel, w.n, w.indptr, w.indices, w.values, w.X, w.W)
        assert np.array_equal(rd.take(w.n * d_out, np.float64), Y.ravel())
        assert np.array_equal(rd.take(w.n * d_out, np.float64), S.ravel())
        assert rd.done()


def test_sanitized_column_sampler(prog, tmp_path):
    """Sparse rows (sorted list), dense rows (bitmap) and rows past half of the columns (complement drawn)."""
    rng = np.random.default_rng(3)
    for n_cols in (1, 63, 64, 65, 1000):
        deg = rng.integers(0, n_cols + 1, 40)
        deg[:4] = [0, n_cols, min(1, n_cols), n_cols // 2 + 1]
        indptr = np.zeros(41, dtype=np.int64); np.cumsum(deg, out=indptr[1:])
        raw = run(prog, "cols", [40, n_cols, int(indptr[-1]), 12345, 0, 0], [indptr], tmp_path)
        rd = Reader(raw)
        assert int(rd.take(1, np.int64)[0]) == 0
        got = rd.take(int(indptr[-1]), np.int32)
        assert rd.done()
        ip2, want = workloads.sample_columns(deg, n_cols, 12345)
        assert np.array_equal(ip2, indptr) and np.array_equal(got, want)
        for r in range(40):
            row = got[indptr[r]:indptr[r + 1]]
            assert (np.diff(row) > 0).all() and (row.size == 0 or (row[0] >= 0 and row[-1] < n_cols))


# ------------------------------------------------------------------------------------------- property test

@st.composite
def csr_and_format(draw):
    n_rows = draw(st.integers(1, 24))
    n_cols = draw(st.integers(1, 40))
    c = draw(st.integers(1, min(n_cols + 2, 9)))
    k = draw(st.integers(0, 6))
    rows = draw(st.lists(st.lists(st.integers(0, n_cols - 1), max_size=n_cols, unique=True).map(sorted),
                         min_size=n_rows, max_size=n_rows))
    seed = draw(st.integers(0, 2**31 - 1))
    return n_rows, n_cols, c, k, rows, seed


@settings(max_examples=150, deadline=None, suppress_health_check=[HealthCheck.too_slow, HealthCheck.data_too_large])
@given(csr_and_format())
def test_property_hyb_is_valid_and_its_spmm_is_the_definition(case):
    n_rows, n_cols, c, k, rows, seed = case
    indptr = np.zeros(n_rows + 1, dtype=np.int32)
    indptr[1:] = np.cumsum([len(r) for r in rows])
    indices = np.array([j for r in rows for j in r], dtype=np.int32)
    rng = np.random.default_rng(seed)
    values = rng.standard_normal(indices.shape[0]).astype(np.float32)
    values[values == 0] = 1.0
    X = rng.standard_normal((n_cols, 3)).astype(np.float32)
    h = oracle.hyb_build(n_rows, n_cols, indptr, indices, values, c, k)
    stats = decode_and_check(h, n_rows, n_cols, indptr, indices, values)
    assert stats is not None
    Y, S = oracle.spmm_csr(n_rows, indptr, indices, values, X)
    Yh = oracle.spmm_hyb(h, X)
    # the same fp64 products in another order (pads add +0.0): a few ulps of the magnitude sum
    assert (np.abs(Yh - Y) <= 1e-13 * S + 0.0).all()
    assert (Yh[np.diff(indptr) == 0] == 0).all()
