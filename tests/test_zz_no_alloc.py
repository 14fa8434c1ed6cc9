"""sptir_spmm_noalloc (the entry point for callers that cannot allocate): its Y
must equal sptir_spmm's bit for bit (same kernels, same summation order; only the
place of the heavy pieces' partial sums differs) and meet the oracle's bar, on two
calls in a row, the second on a smaller input, so that what the first call left in
the static scratch is seen to be harmless."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_helpers import assert_y_close, upload

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def hub_workload(seed, n_rows, n_cols, feat, n_hubs, hub_deg):
    rng = np.random.default_rng(seed)
    deg = np.minimum(rng.geometric(0.1, n_rows), n_cols)
    deg[rng.choice(n_rows, size=n_hubs, replace=False)] = hub_deg
    return workloads.random_csr(n_rows, n_cols, deg, seed, feat)


def run_both(sptir, w, c, k):
    d = upload(w)
    hyb = sptir.sptir_hyb_build(w.n_rows, w.n_cols, d.indptr, d.indices, d.values, c, k)
    info = sptir.sptir_hyb_info(hyb)
    Y_ref = torch.full((w.n_rows, w.feat), float("nan"), device="cuda")
    Y_new = torch.full((w.n_rows, w.feat), float("nan"), device="cuda")
    sptir.sptir_spmm(hyb, d.X, Y_ref)
    sptir.sptir_spmm_noalloc(hyb, d.X, Y_new)
    torch.cuda.synchronize()
    return info, Y_ref.cpu().numpy(), Y_new.cpu().numpy()


def test_noalloc_matches_spmm_twice_in_a_row(gpu_lib):
    sptir = gpu_lib
    # first call: 12 hub rows of 9,000 non-zeros (24 heavy pieces in about 54 heavy lists); second call: a smaller
    # matrix with 3 hub rows, so it reads only the front of what the first call wrote to the scratch
    cases = [(11, 3000, 12000, 96, 12, 9000, 2, 4), (12, 900, 5000, 40, 3, 4100, 1, 3)]
    for seed, n_rows, n_cols, feat, n_hubs, hub_deg, c, k in cases:
        say(f"[noalloc] seed={seed} n_rows={n_rows} n_cols={n_cols} feat={feat} hubs={n_hubs}x{hub_deg} c={c} k={k}")
        w = hub_workload(seed, n_rows, n_cols, feat, n_hubs, hub_deg)
        info, Y_ref, Y_new = run_both(sptir, w, c, k)
        assert info["n_heavy_pieces"] >= n_hubs, "the case must exercise the partial-sum scratch"
        assert np.array_equal(Y_ref.view(np.uint32), Y_new.view(np.uint32)), "sptir_spmm_noalloc differs from sptir_spmm"
        Yo, So = oracle.spmm_csr(w.n_rows, w.indptr, w.indices, w.values, w.X)
        assert_y_close(Y_new, Yo, So, what=f"noalloc seed {seed}")


def test_noalloc_without_long_rows_and_on_named_config(gpu_lib):
    sptir = gpu_lib
    w = workloads.make_config("small")      # one hub row of 19,716 non-zeros
    info, Y_ref, Y_new = run_both(sptir, w, w.n_col_parts, w.max_bucket_log2)
    assert info["n_heavy_pieces"] >= 1
    assert np.array_equal(Y_ref.view(np.uint32), Y_new.view(np.uint32))
    w = workloads.make_config("tiny")
    info, Y_ref, Y_new = run_both(sptir, w, w.n_col_parts, w.max_bucket_log2)
    assert np.array_equal(Y_ref.view(np.uint32), Y_new.view(np.uint32))
    Yo, So = oracle.spmm_csr(w.n_rows, w.indptr, w.indices, w.values, w.X)
    assert_y_close(Y_new, Yo, So, what="noalloc tiny")


def test_noalloc_refuses_what_the_scratch_cannot_hold(gpu_lib):
    sptir = gpu_lib
    # 9,000 rows of 2,100 non-zeros in one partition: 9,000 heavy pieces (+ about 18,500 heavy lists) x 128 floats x 4 bytes
    # = 14 MB of partial sums, more than the 8 MiB of static scratch
    deg = np.full(9000, 2100, dtype=np.int64)
    w = workloads.random_csr(9000, 8192, deg, 5, 32)
    d = upload(w)
    hyb = sptir.sptir_hyb_build(w.n_rows, w.n_cols, d.indptr, d.indices, d.values, 1, 3)
    info = sptir.sptir_hyb_info(hyb)
    assert info["n_heavy_pieces"] == 9000
    assert (info["n_heavy_pieces"] + info["n_heavy_lists"]) * 128 * 4 > 8 * 1024 * 1024
    Y = torch.zeros(w.n_rows, w.feat, device="cuda")
    with pytest.raises(sptir.SptirError) as e:
        sptir.sptir_spmm_noalloc(hyb, d.X, Y)
    assert e.value.status == 6 and "static scratch" in str(e.value)
    torch.cuda.synchronize()
    assert (Y == 0).all(), "a refused call must not have enqueued anything"
    # the allocating entry point serves it
    sptir.sptir_spmm(hyb, d.X, Y)
    torch.cuda.synchronize()
    Yo, So = oracle.spmm_csr(w.n_rows, w.indptr, w.indices, w.values, w.X)
    assert_y_close(Y.cpu().numpy(), Yo, So, what="through sptir_spmm")
    # half the rows fit, on the same GPU right after
    w2 = workloads.random_csr(4000, 8192, deg[:4000], 6, 32)
    d2 = upload(w2)
    hyb2 = sptir.sptir_hyb_build(w2.n_rows, w2.n_cols, d2.indptr, d2.indices, d2.values, 1, 3)
    Ya = torch.empty(w2.n_rows, 32, device="cuda"); Yb = torch.empty(w2.n_rows, 32, device="cuda")
    sptir.sptir_spmm_noalloc(hyb2, d2.X, Ya)
    sptir.sptir_spmm(hyb2, d2.X, Yb)
    torch.cuda.synchronize()
    assert torch.equal(Ya, Yb)
