"""Seeded random matrices, formats and launch plans: for every case the hyb arrays must equal the oracle's bit for
bit and sptir_spmm must agree with the fp64 definition to the parity bar; every fifth case the stream that
sptir_spmm reads is decoded on the host as well.  The parametrised tests fix the shapes a reader can reason about;
this one walks the combinations nobody wrote down (empty rows next to rows as long as the matrix is wide, one value
per row or not, any c and k, every build option at once)."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_helpers import assert_y_close, fetch_hyb, upload
from hyb_checks import assert_same_hyb
import test_gpu_stream as stream_test

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def random_case(rng):
    n_rows = int(rng.integers(1, 6000))
    n_cols = int(rng.integers(1, 6000))
    feat = int(rng.choice([1, 3, 4, 8, 16, 30, 32, 64, 96, 128, 130, 256, 384]))
    kind = rng.integers(0, 4)
    if kind == 0:
        deg = rng.geometric(0.2, n_rows)
    elif kind == 1:
        deg = (rng.pareto(1.1, n_rows) * 4).astype(np.int64) + 1
    elif kind == 2:
        deg = rng.integers(0, min(n_cols, 300) + 1, n_rows)
    else:
        deg = rng.geometric(0.3, n_rows)
        for r in rng.choice(n_rows, size=min(n_rows, 4), replace=False):
            deg[r] = n_cols
    deg[rng.random(n_rows) < rng.random() * 0.5] = 0
    w = workloads.random_csr(n_rows, n_cols, np.minimum(deg, n_cols), int(rng.integers(1 << 30)), feat)
    if rng.random() < 0.3 and w.nnz:
        w.values[:] = np.repeat(rng.standard_normal(n_rows).astype(np.float32), np.diff(w.indptr))
    c = int(rng.choice([1, 2, 3, 5, 8, 16, 33]))
    k = int(rng.choice([0, 1, 3, 5, 8, 11]))
    opts = {"feat_hint": feat}
    if rng.random() < 0.5:
        opts["rounds"] = int(rng.choice([1, 2]))
    if rng.random() < 0.4:
        opts["heavy_len"] = int(rng.choice([1, 7, 16, 63, 64, 65, 200, 1000]))
    if rng.random() < 0.3:
        opts["row_block"] = int(rng.choice([8, 16, 32, 64, 128, 256]))
    if rng.random() < 0.2:
        opts["wide_stream"] = 1
    if rng.random() < 0.2:
        opts["full_rows"] = 1
    if rng.random() < 0.2:
        opts["keep_values"] = 1
    if rng.random() < 0.3:
        opts["sweep_kb"] = int(rng.choice([1, 64, 512, 4096]))
    if opts.get("rounds") == 2 and rng.random() < 0.7:
        opts["parts_per_launch"] = int(rng.integers(1, c + 1))
    return w, c, k, opts


@pytest.mark.parametrize("seed", [2207, 4606])
def test_random_matrices_formats_and_plans(gpu_lib, seed):
    sptir = gpu_lib
    rng = np.random.default_rng(seed)
    for case in range(120):
        w, c, k, opts = random_case(rng)
        say(f"[random {seed}/{case}] rows={w.n_rows} cols={w.n_cols} nnz={w.nnz} feat={w.feat} c={c} k={k} {opts}")
        d = upload(w)
        hyb = sptir.sptir_hyb_build_ex(w.n_rows, w.n_cols, d.indptr, d.indices, d.values, c, k, opts)
        got, info = fetch_hyb(sptir, hyb)
        assert_same_hyb(got, oracle.hyb_build(w.n_rows, w.n_cols, w.indptr, w.indices, w.values, c, k))
        Y = torch.full((w.n_rows, w.feat), float("nan"), device="cuda")
        sptir.sptir_spmm(hyb, d.X, Y)
        Yr, Sr = oracle.spmm_csr(w.n_rows, w.indptr, w.indices, w.values, w.X)
        assert_y_close(Y.cpu().numpy(), Yr, Sr, what=f"seed {seed} case {case}")
        if case % 5 == 0 and w.nnz < 300000:
            rows, cols, _ = stream_test.decode(sptir, hyb, info, w)
            want = np.repeat(np.arange(w.n_rows, dtype=np.int64), np.diff(w.indptr)) * w.n_cols + w.indices
            assert np.array_equal(np.sort(rows * w.n_cols + cols), want), "the stream's entries are not those of A"
        hyb.destroy()
