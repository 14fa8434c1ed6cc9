"""GPU parity tests of SDDMM on CSR: through the C ABI, against the fp64 oracle.
Criterion: |B_gpu - B_oracle| <= 1e-5 * |a_ij| * sum_k |x_ik y_kj| per entry (fp32 products and a d-term sum
against fp64: the error is a few u * sqrt(d) of that magnitude sum, u = 2^-24), and exactly 0 where it is 0."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from test_gpu_parity import ragged_workload, say

pytestmark = pytest.mark.gpu
B_TOL = 1e-5


def run_sddmm(sptir, w, Xr, Yt, in_place=False):
    dev = "cuda"
    ip = torch.from_numpy(w.indptr).to(dev)
    ix = torch.from_numpy(w.indices).to(dev)
    va = torch.from_numpy(w.values).to(dev)
    B = va if in_place else torch.full((w.nnz,), float("nan"), device=dev)
    sptir.sptir_sddmm_csr(w.n_rows, w.n_cols, ip, ix, va, torch.from_numpy(Xr).to(dev), torch.from_numpy(Yt).to(dev), B)
    return B.cpu().numpy()


def assert_b_close(B_gpu, B_ref, M_ref, what):
    B_gpu = B_gpu.astype(np.float64)
    assert np.isfinite(B_gpu).all(), f"{what}: non-finite output"
    zero = M_ref == 0
    assert (B_gpu[zero] == 0).all(), what
    ratio = np.abs(B_gpu - B_ref)[~zero] / M_ref[~zero]
    worst = float(ratio.max()) if ratio.size else 0.0
    assert worst <= B_TOL, f"{what}: max normalised error {worst:.3e}"
    return worst


def left_operand(w, feat, seed):
    return np.random.default_rng(seed).standard_normal((w.n_rows, feat)).astype(np.float32)


@pytest.mark.parametrize("feat", [1, 3, 4, 8, 28, 32, 36, 64, 100, 128, 132, 256, 260, 512, 516, 640])
def test_sddmm_feature_widths(gpu_lib, feat):
    say(f"[sddmm feat] feat={feat}")
    w = ragged_workload(700 + feat, 1300, 1100, feat, max_deg=700, long_rows=5)
    Xr = left_operand(w, feat, feat)
    B = run_sddmm(gpu_lib, w, Xr, w.X)
    Br, Mr = oracle.sddmm_csr(w.n_rows, w.indptr, w.indices, w.values, Xr, w.X)
    assert_b_close(B, Br, Mr, f"feat={feat}")


def test_sddmm_in_place_and_repeatable(gpu_lib):
    w = ragged_workload(41, 900, 1000, 64, max_deg=500, long_rows=3)
    Xr = left_operand(w, 64, 1)
    B1 = run_sddmm(gpu_lib, w, Xr, w.X)
    B2 = run_sddmm(gpu_lib, w, Xr, w.X, in_place=True)     # B written over A's values
    assert np.array_equal(B1, B2)


def test_sddmm_many_empty_rows_and_tiny_inputs(gpu_lib):
    # mostly empty rows: the row of an entry is found by walking indptr
    rng = np.random.default_rng(5)
    deg = np.zeros(5000, dtype=np.int64)
    deg[rng.choice(5000, 40, replace=False)] = rng.integers(1, 300, 40)
    w = workloads.random_csr(5000, 700, deg, 5, 32)
    Xr = left_operand(w, 32, 2)
    Br, Mr = oracle.sddmm_csr(w.n_rows, w.indptr, w.indices, w.values, Xr, w.X)
    assert_b_close(run_sddmm(gpu_lib, w, Xr, w.X), Br, Mr, "empty rows")
    # one entry; and no entries at all (nothing is launched)
    w1 = workloads.random_csr(3, 4, np.array([0, 1, 0]), 1, 8)
    X1 = left_operand(w1, 8, 3)
    Br, Mr = oracle.sddmm_csr(3, w1.indptr, w1.indices, w1.values, X1, w1.X)
    assert_b_close(run_sddmm(gpu_lib, w1, X1, w1.X), Br, Mr, "single entry")
    w0 = workloads.random_csr(3, 4, np.array([0, 0, 0]), 1, 8)
    assert run_sddmm(gpu_lib, w0, left_operand(w0, 8, 4), w0.X).shape == (0,)


def test_sddmm_closed_forms(gpu_lib):
    w = ragged_workload(43, 600, 800, 128, max_deg=300, long_rows=2)
    ones_r, ones_c = np.ones((w.n_rows, 128), np.float32), np.ones((w.n_cols, 128), np.float32)
    assert np.array_equal(run_sddmm(gpu_lib, w, ones_r, ones_c), 128.0 * w.values)      # exact in fp32
    rng = np.random.default_rng(3)
    lab_r, lab_c = rng.integers(0, 128, w.n_rows), rng.integers(0, 128, w.n_cols)
    B = run_sddmm(gpu_lib, w, np.eye(128, dtype=np.float32)[lab_r], np.eye(128, dtype=np.float32)[lab_c])
    rows = np.repeat(np.arange(w.n_rows), np.diff(w.indptr))
    assert np.array_equal(B, np.where(lab_r[rows] == lab_c[w.indices], w.values, np.float32(0)))


def test_sddmm_unaligned_views(gpu_lib):
    w = ragged_workload(47, 300, 350, 12, max_deg=200, long_rows=2)
    Xr = left_operand(w, 12, 5)
    Br, Mr = oracle.sddmm_csr(w.n_rows, w.indptr, w.indices, w.values, Xr, w.X)
    dev = "cuda"
    ip, ix, va = (torch.from_numpy(a).to(dev) for a in (w.indptr, w.indices, w.values))
    for shift in (1, 2):
        xb = torch.empty(Xr.size + 4, device=dev)
        yb = torch.empty(w.X.size + 4, device=dev)
        X = xb[shift:shift + Xr.size].view(w.n_rows, 12); X.copy_(torch.from_numpy(Xr))
        Y = yb[shift:shift + w.X.size].view(w.n_cols, 12); Y.copy_(torch.from_numpy(w.X))
        B = torch.full((w.nnz,), float("nan"), device=dev)
        gpu_lib.sptir_sddmm_csr(w.n_rows, w.n_cols, ip, ix, va, X, Y, B)
        assert_b_close(B.cpu().numpy(), Br, Mr, f"shift={shift}")


def test_sddmm_error_paths(gpu_lib):
    w = ragged_workload(48, 50, 60, 8, max_deg=20)
    dev = "cuda"
    ip, ix, va = (torch.from_numpy(a).to(dev) for a in (w.indptr, w.indices, w.values))
    X = torch.zeros(w.n_rows, 8, device=dev); Y = torch.zeros(w.n_cols, 8, device=dev)
    with pytest.raises(ValueError):
        gpu_lib.sptir_sddmm_csr(w.n_rows, w.n_cols, ip, ix, va, X, Y[:, :4].contiguous(), torch.empty(w.nnz, device=dev))
    with pytest.raises(ValueError):
        gpu_lib.sptir_sddmm_csr(w.n_rows, w.n_cols, ip, ix, va, X, Y, torch.empty(w.nnz + 1, device=dev))
    with pytest.raises(gpu_lib.SptirError):      # B overlapping a dense operand
        gpu_lib.sptir_sddmm_csr(w.n_rows, w.n_cols, ip, ix, va, X, Y, X.view(-1)[:w.nnz])


@pytest.mark.parametrize("name", ["tiny", "small", "medium", "protein", "social"])
def test_sddmm_named_configs(gpu_lib, name):
    w = workloads.make_config(name, feat=128 if name == "social" else None)
    say(f"[sddmm config] {name} nnz={w.nnz} feat={w.feat}")
    Xr = left_operand(w, w.feat, 9)
    B = run_sddmm(gpu_lib, w, Xr, w.X)
    Br, Mr = oracle.sddmm_csr(w.n_rows, w.indptr, w.indices, w.values, Xr, w.X)
    worst = assert_b_close(B, Br, Mr, name)
    say(f"[sddmm config] {name}: max_err={worst:.2e}")


def run_sddmm_plan(sptir, w, Xr, Yt, c, feat_hint=0, in_place=False):
    dev = "cuda"
    ip = torch.from_numpy(w.indptr).to(dev)
    ix = torch.from_numpy(w.indices).to(dev)
    va = torch.from_numpy(w.values).to(dev)
    plan = sptir.sptir_sddmm_plan_build(w.n_rows, w.n_cols, ip, ix, c, feat_hint)
    info = sptir.sptir_sddmm_plan_info(plan)
    B = va if in_place else torch.full((w.nnz,), float("nan"), device=dev)
    sptir.sptir_sddmm(plan, va, torch.from_numpy(Xr).to(dev), torch.from_numpy(Yt).to(dev), B)
    out = B.cpu().numpy()
    plan.destroy()
    return out, info


@pytest.mark.parametrize("c", [1, 2, 3, 8, 16, 40, 2000])
@pytest.mark.parametrize("feat", [4, 32, 100, 128, 7])
def test_sddmm_with_plan_equals_csr_order(gpu_lib, c, feat):
    """Partition order changes where an entry is computed, not how: the plan path must give the very bits of the
    CSR-order kernel (same per-entry arithmetic), for any number of partitions including more than columns."""
    say(f"[sddmm plan] c={c} feat={feat}")
    w = ragged_workload(800 + feat, 1300, 1100, feat, max_deg=700, long_rows=5)
    Xr = left_operand(w, feat, feat)
    want = run_sddmm(gpu_lib, w, Xr, w.X)
    got, info = run_sddmm_plan(gpu_lib, w, Xr, w.X, c)
    assert info["n_col_parts"] == min(c, w.n_cols) and info["nnz"] == w.nnz
    assert np.array_equal(got, want)
    Br, Mr = oracle.sddmm_csr(w.n_rows, w.indptr, w.indices, w.values, Xr, w.X)
    assert_b_close(got, Br, Mr, f"plan c={c} feat={feat}")


def test_sddmm_plan_edge_cases(gpu_lib):
    dev = "cuda"
    # no entries
    w0 = workloads.random_csr(3, 4, np.array([0, 0, 0]), 1, 8)
    got, info = run_sddmm_plan(gpu_lib, w0, left_operand(w0, 8, 4), w0.X, 2)
    assert got.shape == (0,) and info["nnz"] == 0
    # in place, automatic partition count, repeatable
    w = ragged_workload(49, 2000, 2500, 64, max_deg=1200, long_rows=10)
    Xr = left_operand(w, 64, 1)
    a, info = run_sddmm_plan(gpu_lib, w, Xr, w.X, 0, feat_hint=64)
    b, _ = run_sddmm_plan(gpu_lib, w, Xr, w.X, 0, feat_hint=64, in_place=True)
    assert np.array_equal(a, b) and info["n_col_parts"] in (1,) + tuple(range(8, 1025, 8))
    with pytest.raises(gpu_lib.SptirError):       # negative partition count
        gpu_lib.sptir_sddmm_plan_build(w.n_rows, w.n_cols, torch.from_numpy(w.indptr).to(dev),
                                       torch.from_numpy(w.indices).to(dev), -1)


@pytest.mark.parametrize("name", ["medium", "protein", "social"])
def test_sddmm_plan_named_configs(gpu_lib, name):
    w = workloads.make_config(name, feat=128)
    Xr = left_operand(w, 128, 9)
    B, info = run_sddmm_plan(gpu_lib, w, Xr, w.X, 0, feat_hint=128)
    say(f"[sddmm plan config] {name}: c={info['n_col_parts']} runs={info['n_runs']} bytes={info['device_bytes']}")
    Br, Mr = oracle.sddmm_csr(w.n_rows, w.indptr, w.indices, w.values, Xr, w.X)
    assert_b_close(B, Br, Mr, name)
