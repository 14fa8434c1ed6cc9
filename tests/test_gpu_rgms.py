"""GPU parity tests of the relational gather-matmul-scatter operator: through the C ABI, against the fp64 oracle.
Criterion: |Y_gpu - Y_oracle| <= 1e-5 * sum |a x w| per element of Y (float32 products and sums, the
contributions meeting in float atomic adds in any order), and exactly 0 where that sum is 0.  The 3-D hyb arrays
(the hyb(1, k) of the stacked matrix) are covered bit for bit by the builder tests; here the operator is checked."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from test_gpu_parity import say

pytestmark = pytest.mark.gpu
Y_TOL = 1e-5


def run_rgms(sptir, w, k=-1, workspace_d_out=0, repeat=1):
    dev = "cuda"
    ip = torch.from_numpy(w.indptr).to(dev)
    ix = torch.from_numpy(w.indices).to(dev)
    va = torch.from_numpy(w.values).to(dev)
    h = sptir.sptir_rgms_build(w.n_rel, w.n, w.n, ip, ix, va, k, workspace_d_out)
    info = sptir.sptir_rgms_info(h)
    X, W = torch.from_numpy(w.X).to(dev), torch.from_numpy(w.W).to(dev)
    outs = []
    for _ in range(repeat):
        Y = torch.full((w.n, w.W.shape[2]), float("nan"), device=dev)
        sptir.sptir_rgms(h, X, W, Y)
        outs.append(Y.cpu().numpy())
    h.destroy()
    return (outs[0] if repeat == 1 else outs), info


def assert_y_close(Y_gpu, Y_ref, S_ref, what):
    Y_gpu = Y_gpu.astype(np.float64)
    assert np.isfinite(Y_gpu).all(), f"{what}: non-finite output"
    zero = S_ref == 0
    assert (Y_gpu[zero] == 0).all(), what
    ratio = np.abs(Y_gpu - Y_ref)[~zero] / S_ref[~zero]
    worst = float(ratio.max()) if ratio.size else 0.0
    assert worst <= Y_TOL, f"{what}: max normalised error {worst:.3e}"
    return worst


@pytest.mark.parametrize("d_in,d_out", [(32, 32), (32, 64), (64, 32), (128, 96), (64, 128)])
@pytest.mark.parametrize("k", [-1, 0, 2, 5])
@pytest.mark.parametrize("workspace", [0, 64, 128])
def test_rgms_small_graphs(gpu_lib, d_in, d_out, k, workspace):
    """workspace 0: atomics only; 64: the workspace serves d_out <= 64 and the wider calls fall back to atomics."""
    say(f"[rgms] d_in={d_in} d_out={d_out} k={k} workspace={workspace}")
    w = workloads.make_hetero("hetero_tiny", seed=d_in + d_out + k, d_in=d_in, d_out=d_out)
    Y, info = run_rgms(gpu_lib, w, k, workspace)
    assert info["nnz"] == w.nnz and info["n_relations"] == w.n_rel and info["max_bucket_log2"] == (5 if k < 0 else k)
    assert info["workspace_d_out"] == workspace
    Yr, Sr = oracle.rgms(w.n_rel, w.n, w.indptr, w.indices, w.values, w.X, w.W)
    assert_y_close(Y, Yr, Sr, f"d_in={d_in} d_out={d_out} k={k}")


def test_rgms_long_rows_and_empty_relations(gpu_lib):
    """One (relation, row) pair with thousands of entries (several remainder tiles), relations without entries,
    rows without entries."""
    rng = np.random.default_rng(4)
    n, n_rel = 2500, 6
    trip = set()
    for j in rng.choice(n, 2300, replace=False):
        trip.add((1, 17, int(j)))                       # a very long stacked row
    for _ in range(4000):
        trip.add((int(rng.choice([0, 1, 4])), int(rng.integers(0, n // 2)), int(rng.integers(0, n))))   # 2, 3, 5 empty
    key = np.array(sorted((r * n + i) * n + j for r, i, j in trip), dtype=np.int64)
    stacked = key // n
    counts = np.bincount(stacked, minlength=n_rel * n)
    indptr = np.zeros(n_rel * n + 1, dtype=np.int64); np.cumsum(counts, out=indptr[1:])
    w = workloads.HeteroWorkload("long", n, n_rel, indptr.astype(np.int32), (key % n).astype(np.int32),
                                 rng.uniform(-1, 1, key.shape[0]).astype(np.float32),
                                 rng.standard_normal((n, 32)).astype(np.float32),
                                 rng.standard_normal((n_rel, 32, 32)).astype(np.float32))
    Yr, Sr = oracle.rgms(n_rel, n, w.indptr, w.indices, w.values, w.X, w.W)
    for workspace in (0, 32):
        Y, info = run_rgms(gpu_lib, w, workspace_d_out=workspace)
        assert_y_close(Y, Yr, Sr, f"long rows workspace={workspace}")


def test_rgms_reduces_to_spmm(gpu_lib):
    """One relation and W = I: the operator is Y = A X; 0/1 products are exact, so only the summation order differs."""
    w0 = workloads.make_config("small")
    n, feat = w0.n_rows, 32
    rng = np.random.default_rng(2)
    X = rng.standard_normal((n, feat)).astype(np.float32)
    w = workloads.HeteroWorkload("single", n, 1, w0.indptr, w0.indices, w0.values, X, np.eye(feat, dtype=np.float32)[None])
    Yr, Sr = oracle.spmm_csr(n, w0.indptr, w0.indices, w0.values, X)
    for workspace in (0, 32):
        Y, info = run_rgms(gpu_lib, w, workspace_d_out=workspace)
        assert_y_close(Y, Yr, Sr, f"single relation workspace={workspace}")


def test_rgms_edge_cases_and_errors(gpu_lib):
    dev = "cuda"
    # no entries at all: Y is still overwritten with zeros
    ip = torch.zeros(3 * 10 + 1, dtype=torch.int32, device=dev)
    ix = torch.zeros(0, dtype=torch.int32, device=dev); va = torch.zeros(0, device=dev)
    h = gpu_lib.sptir_rgms_build(3, 10, 10, ip, ix, va)
    Y = torch.full((10, 32), float("nan"), device=dev)
    gpu_lib.sptir_rgms(h, torch.zeros(10, 32, device=dev), torch.zeros(3, 32, 32, device=dev), Y)
    assert (Y == 0).all()
    with pytest.raises(gpu_lib.SptirError):        # feature sizes the matrix-core path does not cover
        gpu_lib.sptir_rgms(h, torch.zeros(10, 48, device=dev), torch.zeros(3, 48, 32, device=dev), Y)
    with pytest.raises(ValueError):
        gpu_lib.sptir_rgms(h, torch.zeros(10, 32, device=dev), torch.zeros(2, 32, 32, device=dev), Y)
    with pytest.raises(gpu_lib.SptirError):        # a bucket count beyond what the builder supports
        gpu_lib.sptir_rgms_build(7, 10, 10, torch.zeros(7 * 10 + 1, dtype=torch.int32, device=dev), ix, va, 9)
    with pytest.raises(gpu_lib.SptirError):        # workspace width not a multiple of 32
        gpu_lib.sptir_rgms_build(3, 10, 10, ip, ix, va, -1, 48)
    h.destroy()


def capped_hetero(seed, n, n_rel, cap, d=32):
    """A heterogeneous graph whose every (relation, row) pair has between 0 and `cap` entries."""
    rng = np.random.default_rng(seed)
    counts = rng.integers(0, cap + 1, n_rel * n)
    counts[rng.random(n_rel * n) < 0.5] = 0
    counts[rng.integers(0, n_rel * n, 8)] = cap          # the cap is reached
    indptr = np.zeros(n_rel * n + 1, dtype=np.int64); np.cumsum(counts, out=indptr[1:])
    indices = np.concatenate([np.sort(rng.choice(n, int(m), replace=False)) for m in counts if m] or [np.zeros(0)])
    return workloads.HeteroWorkload("capped", n, n_rel, indptr.astype(np.int32), indices.astype(np.int32),
                                    rng.uniform(-1, 1, indices.shape[0]).astype(np.float32),
                                    rng.standard_normal((n, d)).astype(np.float32),
                                    rng.standard_normal((n_rel, d, d)).astype(np.float32))


def test_rgms_workspace_path_is_reproducible(gpu_lib):
    """With the workspace, and no (relation, row) pair longer than the widest bucket (so nothing goes to the
    remainder, whose pieces meet in atomic adds), every sum has a fixed order: calls agree bit for bit."""
    wl = capped_hetero(9, 700, 5, 32)
    assert np.diff(wl.indptr).max() == 32
    (Y1, Y2, Y3), info = run_rgms(gpu_lib, wl, workspace_d_out=32, repeat=3)
    assert info["max_bucket_log2"] == 5
    assert np.array_equal(Y1, Y2) and np.array_equal(Y1, Y3)
    Yr, Sr = oracle.rgms(wl.n_rel, wl.n, wl.indptr, wl.indices, wl.values, wl.X, wl.W)
    assert_y_close(Y1, Yr, Sr, "capped workspace")
    # and on a graph with remainder pieces the two paths agree with the oracle to rounding
    w = workloads.make_hetero("hetero_a")
    assert np.diff(w.indptr).max() > 32
    Ya, _ = run_rgms(gpu_lib, w, workspace_d_out=0)
    Yb, _ = run_rgms(gpu_lib, w, workspace_d_out=32)
    Yr, Sr = oracle.rgms(w.n_rel, w.n, w.indptr, w.indices, w.values, w.X, w.W)
    assert_y_close(Ya, Yr, Sr, "atomics"); assert_y_close(Yb, Yr, Sr, "workspace")


@pytest.mark.parametrize("workspace", [0, 32])
@pytest.mark.parametrize("name", ["hetero_a", "hetero_b", "hetero_c", "hetero_d", "hetero_e"])
def test_rgms_named_configs(gpu_lib, name, workspace):
    w = workloads.make_hetero(name)
    Y, info = run_rgms(gpu_lib, w, workspace_d_out=workspace)
    say(f"[rgms config] {name}: nnz={w.nnz} pairs={info['n_stacked_rows_stored']} pads={info['n_pad_slots']} "
        f"tiles={info['n_tiles']}")
    Yr, Sr = oracle.rgms(w.n_rel, w.n, w.indptr, w.indices, w.values, w.X, w.W)
    worst = assert_y_close(Y, Yr, Sr, name)
    say(f"[rgms config] {name}: max_err={worst:.2e}")
