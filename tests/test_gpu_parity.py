"""GPU parity tests: every call goes through the C ABI (ctypes binding) and is
compared with the CPU oracle on the same seeded inputs.  hyb arrays must match
bit for bit; Y within 1e-5 of the oracle, normalised by sum_j |a_ij x_jk|."""
import os

import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_helpers import assert_y_close, fetch_hyb, upload
from hyb_checks import assert_same_hyb, load_golden

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hyb_2_2_example.txt")


def say(msg):
    print(msg, flush=True)


def build_both(sptir, w, c, k, options=None):
    d = upload(w)
    if options:
        hyb = sptir.sptir_hyb_build_ex(w.n_rows, w.n_cols, d.indptr, d.indices, d.values, c, k, options)
    else:
        hyb = sptir.sptir_hyb_build(w.n_rows, w.n_cols, d.indptr, d.indices, d.values, c, k)
    got, info = fetch_hyb(sptir, hyb)
    want = oracle.hyb_build(w.n_rows, w.n_cols, w.indptr, w.indices, w.values, c, k)
    return d, hyb, got, want, info


def ragged_workload(seed, n_rows, n_cols, feat, max_deg, empty_frac=0.15, long_rows=0):
    rng = np.random.default_rng(seed)
    deg = np.minimum(rng.geometric(0.15, n_rows), max_deg)
    deg[rng.random(n_rows) < empty_frac] = 0
    for r in rng.choice(n_rows, size=long_rows, replace=False):
        deg[r] = rng.integers(max_deg // 2, max_deg + 1)
    return workloads.random_csr(n_rows, n_cols, np.minimum(deg, n_cols), seed, feat)


# ------------------------------------------------------------------- builder

def test_hyb_golden_example(gpu_lib):
    g = load_golden(GOLDEN)
    ints = lambda key: np.array(g[key], dtype=np.int32)
    w = workloads.Workload("golden", 5, 12, ints("indptr"), ints("indices"), np.array(g["values"], np.float32),
                           np.ones((12, 1), np.float32), 1, 2, 2)
    d, hyb, got, want, info = build_both(gpu_lib, w, 2, 2)
    assert_same_hyb(got, want)
    for name in ("ell_row", "ell_col", "rem_col", "bucket_slot_ptr"):
        assert np.array_equal(getattr(got, name), np.array(g[name], dtype=getattr(got, name).dtype))
    Y = torch.empty(5, 1, device="cuda")
    gpu_lib.sptir_spmm(hyb, d.X, Y)
    assert np.array_equal(Y.cpu().numpy().ravel(), np.array(g["y_ones"], np.float32))


@pytest.mark.parametrize("seed,n_rows,n_cols,c,k", [
    (0, 300, 300, 1, 0), (1, 777, 513, 1, 5), (2, 1000, 1200, 2, 2), (3, 1025, 999, 3, 1),
    (4, 2500, 2500, 4, 6), (5, 513, 4000, 7, 3), (6, 3000, 64, 16, 2), (7, 255, 700, 100, 3),
    (8, 256, 300, 2, 30), (9, 257, 5000, 5, 9), (10, 1, 50, 2, 2), (11, 4097, 4097, 16, 11)])
def test_hyb_bit_exact_ragged(gpu_lib, seed, n_rows, n_cols, c, k):
    say(f"[hyb ragged] seed={seed} n_rows={n_rows} n_cols={n_cols} c={c} k={k}")
    w = ragged_workload(seed, n_rows, n_cols, 8, max_deg=min(n_cols, 600), long_rows=min(5, n_rows))
    d, hyb, got, want, info = build_both(gpu_lib, w, c, k)
    assert_same_hyb(got, want)
    assert info["nnz"] == w.nnz and info["n_pad_slots"] == want.ell_col.size + want.rem_col.size - w.nnz


def test_hyb_edge_cases(gpu_lib):
    sptir = gpu_lib
    # no non-zeros at all
    w = workloads.random_csr(7, 9, np.zeros(7, np.int64), 0, 4)
    d, hyb, got, want, info = build_both(sptir, w, 3, 2)
    assert_same_hyb(got, want)
    Y = torch.full((7, 4), 5.0, device="cuda")
    sptir.sptir_spmm(hyb, d.X, Y)
    assert (Y == 0).all()
    # zero rows
    w0 = workloads.Workload("z", 0, 5, np.zeros(1, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32),
                            np.ones((5, 3), np.float32), 3, 1, 1)
    d, hyb, got, want, info = build_both(sptir, w0, 2, 1)
    assert_same_hyb(got, want)
    # a full row (every column) and maximum-length pieces
    deg = np.array([64, 0, 64, 1, 33], dtype=np.int64)
    wf = workloads.random_csr(5, 64, deg, 3, 5)
    for c, k in ((1, 6), (1, 5), (2, 5), (4, 3), (64, 0), (3, 0)):
        d, hyb, got, want, info = build_both(sptir, wf, c, k)
        assert_same_hyb(got, want)


def test_hyb_build_is_deterministic(gpu_lib):
    w = workloads.make_config("small")
    d = upload(w)
    a = gpu_lib.sptir_hyb_build(w.n_rows, w.n_cols, d.indptr, d.indices, d.values, 4, 4)
    b = gpu_lib.sptir_hyb_build(w.n_rows, w.n_cols, d.indptr, d.indices, d.values, 4, 4)
    ga, _ = fetch_hyb(gpu_lib, a)
    gb, _ = fetch_hyb(gpu_lib, b)
    assert_same_hyb(ga, gb)


def test_hyb_build_through_torch_allocator(gpu_lib):
    w = workloads.make_config("tiny")
    gpu_lib.sptir_set_allocator(True)
    try:
        d, hyb, got, want, info = build_both(gpu_lib, w, 2, 3)
        assert_same_hyb(got, want)
        hyb.destroy()
    finally:
        gpu_lib.sptir_set_allocator(False)


def test_scratch_blocks_are_kept_and_released(gpu_lib):
    """Under the default allocator the temporaries of a build are kept for the next one: repeated builds (the same
    sizes, then larger and smaller ones) stay bit-exact, and sptir_release_scratch gives the blocks back (free device
    memory does not shrink over the sequence)."""
    gpu_lib.sptir_release_scratch()
    free0, _ = torch.cuda.mem_get_info()
    for n_rows, c, k in ((3000, 4, 5), (3000, 4, 5), (9000, 7, 3), (500, 2, 8), (3000, 4, 5)):
        w = ragged_workload(n_rows, n_rows, n_rows + 100, 8, max_deg=400, long_rows=3)
        d, hyb, got, want, info = build_both(gpu_lib, w, c, k)
        assert_same_hyb(got, want)
        Y = torch.empty(w.n_rows, 8, device="cuda")
        gpu_lib.sptir_spmm(hyb, d.X, Y)
        Yr, Sr = oracle.spmm_csr(w.n_rows, w.indptr, w.indices, w.values, w.X)
        assert_y_close(Y.cpu().numpy(), Yr, Sr, what=f"repeated build {n_rows}")
        hyb.destroy()
        del d, Y
    torch.cuda.synchronize()
    gpu_lib.sptir_release_scratch()
    torch.cuda.empty_cache()
    free1, _ = torch.cuda.mem_get_info()
    assert free1 >= free0 - (64 << 20), f"device memory not given back: {free0} -> {free1}"


def test_torch_allocator_on_a_side_stream(gpu_lib):
    """Build, SpMM and destroy on a side stream with the library's memory coming from torch's allocator, while the
    default stream keeps allocating, filling and freeing blocks of the sizes in play: blocks the library took
    under the side stream must not be handed to the default stream while the side stream still uses them."""
    w = workloads.make_config("small")
    d = upload(w)
    Yr, Sr = oracle.spmm_csr(w.n_rows, w.indptr, w.indices, w.values, w.X)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    gpu_lib.sptir_set_allocator(True)
    try:
        for rep in range(4):
            with torch.cuda.stream(s):
                hyb = gpu_lib.sptir_hyb_build_ex(w.n_rows, w.n_cols, d.indptr, d.indices, d.values, 2, 4,
                                                 {"rounds": 1, "heavy_len": 8}, stream=s)
                Y = torch.empty(w.n_rows, w.feat, device="cuda")
                gpu_lib.sptir_spmm(hyb, d.X, Y, stream=s)
                hyb.destroy()
            for nbytes in (1 << 12, 1 << 16, 1 << 20, 1 << 22):      # default stream: churn
                torch.full((nbytes,), 255, dtype=torch.uint8, device="cuda")
            s.synchronize()
            assert_y_close(Y.cpu().numpy(), Yr, Sr, what=f"torch allocator, side stream, repeat {rep}")
    finally:
        gpu_lib.sptir_set_allocator(False)


def test_error_paths(gpu_lib):
    sptir = gpu_lib
    dev = "cuda"
    t = lambda a, dt: torch.tensor(a, dtype=dt, device=dev)
    vals = t([1.0, 1.0], torch.float32)
    cases = [
        ([0, 2], [2, 1], 2),      # descending columns
        ([0, 2], [1, 1], 2),      # duplicate column
        ([0, 2], [0, 4], 2),      # column out of range
        ([0, 2], [-1, 1], 2),     # negative column
        ([1, 2], [0, 1], 1),      # indptr[0] != 0
        ([0, 1], [0, 1], 1),      # indptr[-1] != nnz
    ]
    for indptr, indices, status in cases:
        with pytest.raises(sptir.SptirError) as e:
            sptir.sptir_hyb_build(1, 4, t(indptr, torch.int32), t(indices, torch.int32), vals, 1, 1)
        assert e.value.status == status, (indptr, indices)
    # decreasing indptr over two rows
    with pytest.raises(sptir.SptirError) as e:
        sptir.sptir_hyb_build(2, 4, t([0, 2, 1], torch.int32), t([0, 1], torch.int32), vals, 1, 1)
    assert e.value.status == 1
    ok = (t([0, 2], torch.int32), t([0, 1], torch.int32), vals)
    for c, k in ((0, 1), (1, -1), (1, 31)):
        with pytest.raises(sptir.SptirError) as e:
            sptir.sptir_hyb_build(1, 4, *ok, c, k)
        assert e.value.status == 1
    hyb = sptir.sptir_hyb_build(1, 4, *ok, 1, 1)
    X = torch.ones(4, 8, device=dev)
    with pytest.raises(sptir.SptirError) as e:      # Y overlapping X
        sptir.sptir_spmm(hyb, X, X[:1])
    assert e.value.status == 1
    # two rows that are legal only because the descent sits on a row boundary
    h2 = sptir.sptir_hyb_build(2, 4, t([0, 1, 2], torch.int32), t([3, 0], torch.int32), vals, 1, 1)
    assert sptir.sptir_hyb_info(h2)["nnz"] == 2


# ---------------------------------------------------------------------- SpMM

@pytest.mark.parametrize("feat", [1, 3, 4, 8, 16, 30, 32, 33, 64, 100, 128, 130, 256, 288])
def test_spmm_feature_widths(gpu_lib, feat):
    say(f"[spmm feat] feat={feat}")
    w = ragged_workload(100 + feat, 1500, 1700, feat, max_deg=900, long_rows=6)
    for c, k in ((1, 3), (3, 5), (4, 10)):
        d, hyb, got, want, info = build_both(gpu_lib, w, c, k)
        Y = torch.full((w.n_rows, feat), float("nan"), device="cuda")
        gpu_lib.sptir_spmm(hyb, d.X, Y)
        Yr, Sr = oracle.spmm_csr(w.n_rows, w.indptr, w.indices, w.values, w.X)
        assert_y_close(Y.cpu().numpy(), Yr, Sr, what=f"feat={feat} c={c} k={k}")


def test_spmm_unaligned_views(gpu_lib):
    w = ragged_workload(7, 400, 500, 12, max_deg=300, long_rows=3)
    d = upload(w)
    hyb = gpu_lib.sptir_hyb_build(w.n_rows, w.n_cols, d.indptr, d.indices, d.values, 2, 4)
    Yr, Sr = oracle.spmm_csr(w.n_rows, w.indptr, w.indices, w.values, w.X)
    for shift in (1, 2):     # X and Y start 4 or 8 bytes past a 16-byte boundary
        xb = torch.empty(w.X.size + 4, device="cuda")
        yb = torch.empty(w.n_rows * 12 + 4, device="cuda")
        X = xb[shift:shift + w.X.size].view(w.n_cols, 12); X.copy_(d.X)
        Y = yb[shift:shift + w.n_rows * 12].view(w.n_rows, 12)
        gpu_lib.sptir_spmm(hyb, X, Y)
        assert_y_close(Y.cpu().numpy(), Yr, Sr, what=f"shift={shift}")


def test_spmm_identity_and_ones(gpu_lib):
    n, feat = 1000, 64
    rng = np.random.default_rng(1)
    X = rng.standard_normal((n, feat)).astype(np.float32)
    dev = "cuda"
    indptr = torch.arange(n + 1, dtype=torch.int32, device=dev)
    indices = torch.arange(n, dtype=torch.int32, device=dev)
    hyb = gpu_lib.sptir_hyb_build(n, n, indptr, indices, torch.ones(n, device=dev), 4, 2)
    Y = torch.empty(n, feat, device=dev)
    Xd = torch.from_numpy(X).to(dev)
    gpu_lib.sptir_spmm(hyb, Xd, Y)
    assert torch.equal(Y, Xd)                     # A = I gives Y = X exactly
    w = ragged_workload(5, 800, 900, 32, max_deg=700, long_rows=4)
    w.values[:] = 1.0
    d = upload(w)
    hyb = gpu_lib.sptir_hyb_build(w.n_rows, w.n_cols, d.indptr, d.indices, d.values, 3, 4)
    Y = torch.empty(w.n_rows, 32, device=dev)
    gpu_lib.sptir_spmm(hyb, torch.ones(w.n_cols, 32, device=dev), Y)
    deg = np.diff(w.indptr).astype(np.float32)     # unit values, X = 1: exactly the degrees
    assert np.array_equal(Y.cpu().numpy(), np.repeat(deg[:, None], 32, 1))


@pytest.mark.parametrize("name", ["tiny", "small", "medium"])
def test_named_configs_full(gpu_lib, name):
    say(f"[config] {name}")
    w = workloads.make_config(name)
    d, hyb, got, want, info = build_both(gpu_lib, w, w.n_col_parts, w.max_bucket_log2)
    assert_same_hyb(got, want)
    Y = torch.empty(w.n_rows, w.feat, device="cuda")
    gpu_lib.sptir_spmm(hyb, d.X, Y)
    Yr, Sr = oracle.spmm_csr(w.n_rows, w.indptr, w.indices, w.values, w.X)
    worst = assert_y_close(Y.cpu().numpy(), Yr, Sr, what=name)
    say(f"[config] {name}: nnz={w.nnz} pads={info['n_pad_slots']} rem_nnz={info['n_rem_nnz']} max_err={worst:.2e}")
    # the no-hyb CSR kernel on the same input
    Y2 = torch.empty_like(Y)
    gpu_lib.sptir_spmm_csr(w.n_rows, w.n_cols, d.indptr, d.indices, d.values, d.X, Y2)
    assert_y_close(Y2.cpu().numpy(), Yr, Sr, what=name + " csr")


@pytest.mark.parametrize("name", ["protein", "social"])
def test_named_configs_full_size_all_rows(gpu_lib, name):
    """Full-size graphs in the launch configuration bench.py times: hyb arrays bit-exact in full, and every
    element of Y against the oracle, at the configuration's own feature size and at the 128 the headline
    measurement uses."""
    say(f"[config] {name}: generating")
    w = workloads.make_config(name)
    say(f"[config] {name}: building on GPU and in the oracle")
    d, hyb, got, want, info = build_both(gpu_lib, w, w.n_col_parts, w.max_bucket_log2)
    assert_same_hyb(got, want)
    del got, want
    for feat in sorted({w.feat, 128}):
        X = w.X if feat == w.feat else np.ascontiguousarray(w.X[:, :feat])
        Y = torch.full((w.n_rows, feat), float("nan"), device="cuda")
        gpu_lib.sptir_spmm(hyb, torch.from_numpy(X).cuda(), Y)
        torch.cuda.synchronize()
        say(f"[config] {name}: oracle on all {w.n_rows} rows at feat={feat}")
        Yr, Sr = oracle.spmm_csr(w.n_rows, w.indptr, w.indices, w.values, X)
        worst = assert_y_close(Y.cpu().numpy(), Yr, Sr, what=f"{name} feat={feat}")
        say(f"[config] {name}: feat={feat} nnz={w.nnz} pads={info['n_pad_slots']} rem_nnz={info['n_rem_nnz']} "
            f"list chunks={info['n_work_items']} heavy pieces={info['n_heavy_pieces']} rounds={info['rounds']} "
            f"max_err={worst:.2e}")
        del Yr, Sr


def test_spmm_csr_ragged(gpu_lib):
    for feat in (5, 32, 96):
        w = ragged_workload(50 + feat, 1200, 1500, feat, max_deg=1000, long_rows=5)
        d = upload(w)
        Y = torch.full((w.n_rows, feat), float("nan"), device="cuda")
        gpu_lib.sptir_spmm_csr(w.n_rows, w.n_cols, d.indptr, d.indices, d.values, d.X, Y)
        Yr, Sr = oracle.spmm_csr(w.n_rows, w.indptr, w.indices, w.values, w.X)
        assert_y_close(Y.cpu().numpy(), Yr, Sr, what=f"csr feat={feat}")


def test_spmm_on_side_stream_and_repeat(gpu_lib):
    w = workloads.make_config("small")
    d, hyb, got, want, info = build_both(gpu_lib, w, 2, 6)
    Yr, Sr = oracle.spmm_csr(w.n_rows, w.indptr, w.indices, w.values, w.X)
    s = torch.cuda.Stream()
    Y = torch.empty(w.n_rows, w.feat, device="cuda")
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        for _ in range(3):                       # Y is overwritten, not accumulated
            gpu_lib.sptir_spmm(hyb, d.X, Y, stream=s)
    s.synchronize()
    assert_y_close(Y.cpu().numpy(), Yr, Sr, what="side stream")


@pytest.mark.parametrize("knobs", [
    {"wide_stream": 1}, {"parts_per_launch": 1}, {"parts_per_launch": 2, "wide_stream": 1},
    {"row_block": 8}, {"row_block": 64, "parts_per_launch": 3}, {"row_block": 128}, {"row_block": 256},
    {"rounds": 1}, {"rounds": 1, "heavy_len": 64}, {"rounds": 1, "heavy_len": 16, "wide_stream": 1},
    {"full_rows": 1}, {"full_rows": 1, "rounds": 1, "heavy_len": 30}, {"full_rows": 1, "wide_stream": 1, "row_block": 32},
    {"full_rows": 1, "row_block": 64}, {"full_rows": 1, "row_block": 128},
    {"rounds": 1, "row_block": 16, "heavy_len": 1}, {"rounds": 2, "parts_per_launch": 1, "heavy_len": 100},
    {"rounds": 2, "heavy_len": 5000}, {"release_canonical": 1, "heavy_len": 70}])
def test_spmm_launch_plan_knobs(gpu_lib, knobs):
    """Every launch plan the builder can choose (record form, partitions per launch, rounds, rows per wavefront,
    which pieces count as heavy) computes the same Y; two runs on one handle agree bit for bit (no atomics
    anywhere on the path)."""
    say(f"[knobs] {knobs}")
    for feat, c, k in ((32, 5, 4), (7, 3, 2), (128, 4, 7)):
        w = ragged_workload(300 + feat, 2300, 2100, feat, max_deg=1500, long_rows=8)
        d = upload(w)
        hyb = gpu_lib.sptir_hyb_build_ex(w.n_rows, w.n_cols, d.indptr, d.indices, d.values, c, k, knobs)
        info = gpu_lib.sptir_hyb_info(hyb)
        if knobs.get("release_canonical"):
            for name in ("ell_col", "ell_val", "rem_col", "rem_val"):
                with pytest.raises(gpu_lib.SptirError) as e:
                    gpu_lib.sptir_hyb_array(hyb, name)
                assert e.value.status == 6
            assert np.array_equal(gpu_lib.sptir_hyb_array(hyb, "ell_row"),
                                  oracle.hyb_build(w.n_rows, w.n_cols, w.indptr, w.indices, w.values, c, k).ell_row)
        else:
            got, _ = fetch_hyb(gpu_lib, hyb)
            assert_same_hyb(got, oracle.hyb_build(w.n_rows, w.n_cols, w.indptr, w.indices, w.values, c, k))
        if "parts_per_launch" in knobs:
            assert info["n_phases"] == -(-c // knobs["parts_per_launch"]) and info["rounds"] == 0
        if knobs.get("rounds") == 1:
            assert info["rounds"] == 1 and info["n_phases"] == 1
        if "row_block" in knobs:
            assert info["row_block"] == knobs["row_block"]
        assert info["full_rows"] == int(knobs.get("full_rows", 0) == 1)
        if "heavy_len" in knobs:
            assert info["heavy_len"] == knobs["heavy_len"]
            lens = np.diff(w.indptr)   # an upper bound: a heavy piece needs a row longer than heavy_len
            assert (info["n_heavy_pieces"] > 0) == bool((lens > knobs["heavy_len"]).any()) or c > 1
        Y = torch.full((w.n_rows, feat), float("nan"), device="cuda")
        gpu_lib.sptir_spmm(hyb, d.X, Y)
        Yr, Sr = oracle.spmm_csr(w.n_rows, w.indptr, w.indices, w.values, w.X)
        assert_y_close(Y.cpu().numpy(), Yr, Sr, what=f"{knobs} feat={feat}")
        Y2 = torch.full((w.n_rows, feat), float("nan"), device="cuda")
        gpu_lib.sptir_spmm(hyb, d.X, Y2)
        assert torch.equal(Y, Y2)


@pytest.mark.parametrize("knobs", [
    {}, {"keep_values": 1}, {"rounds": 1, "heavy_len": 64}, {"rounds": 1, "wide_stream": 1, "heavy_len": 20},
    {"rounds": 2, "parts_per_launch": 1}, {"rounds": 2, "parts_per_launch": 2, "wide_stream": 1, "heavy_len": 300},
    {"row_block": 256}, {"full_rows": 1, "heavy_len": 40}])
def test_spmm_one_value_per_row(gpu_lib, knobs):
    """A matrix whose rows each repeat one value (a row-normalised adjacency matrix) is stored without values in
    the SpMM stream, and the rows of Y are scaled at the end; keep_values turns that off.  Both must meet the
    oracle, in every launch plan."""
    say(f"[one value per row] {knobs}")
    for feat, c, k in ((32, 5, 4), (6, 3, 2), (128, 4, 7), (200, 2, 3)):
        w = ragged_workload(700 + feat, 2300, 2100, feat, max_deg=1500, long_rows=8)
        deg = np.diff(w.indptr)
        per_row = np.random.default_rng(feat).standard_normal(w.n_rows).astype(np.float32)
        w.values[:] = np.repeat(per_row, deg)
        d, hyb, got, want, info = build_both(gpu_lib, w, c, k, dict(knobs) or None)
        assert_same_hyb(got, want)
        assert info["values_per_row"] == (0 if knobs.get("keep_values") else 1)
        Y = torch.full((w.n_rows, feat), float("nan"), device="cuda")
        gpu_lib.sptir_spmm(hyb, d.X, Y)
        Yr, Sr = oracle.spmm_csr(w.n_rows, w.indptr, w.indices, w.values, w.X)
        assert_y_close(Y.cpu().numpy(), Yr, Sr, what=f"one value per row {knobs} feat={feat}")
    # one entry that differs, at the end of a row, and the matrix is stored with its values
    w.values[w.indptr[w.n_rows // 2 + 1] - 1] += 1.0
    d, hyb, got, want, info = build_both(gpu_lib, w, c, k, dict(knobs) or None)
    assert info["values_per_row"] == 0
    Y = torch.full((w.n_rows, feat), float("nan"), device="cuda")
    gpu_lib.sptir_spmm(hyb, d.X, Y)
    Yr, Sr = oracle.spmm_csr(w.n_rows, w.indptr, w.indices, w.values, w.X)
    assert_y_close(Y.cpu().numpy(), Yr, Sr, what=f"almost one value per row {knobs}")


def test_timed_call_and_roof_microbenchmarks(gpu_lib):
    """The measurement aids of the C ABI: sptir_spmm_timed gives the same Y as sptir_spmm and times that add up;
    the roof microbenchmarks return plausible rates and reject bad arguments."""
    sptir = gpu_lib
    w = ragged_workload(5, 3000, 2500, 64, max_deg=1200, long_rows=10)
    d, hyb, got, want, info = build_both(sptir, w, 3, 4, {"rounds": 1, "heavy_len": 64})
    Y = torch.empty(w.n_rows, 64, device="cuda"); Yt = torch.empty_like(Y)
    sptir.sptir_spmm(hyb, d.X, Y)
    t = sptir.sptir_spmm_timed(hyb, d.X, Yt)
    assert torch.equal(Y, Yt)
    assert t["n_list_launches"] >= 1 and t["n_heavy_launches"] >= 1 and t["n_reduce_launches"] == 1
    assert t["ms_lists"] > 0 and t["ms_heavy"] > 0 and t["ms_reduce"] > 0
    X = torch.zeros(4096, 128, device="cuda"); sink = torch.zeros(4, device="cuda")
    ms, nbytes = sptir.sptir_roof_gather(X, 4096, 4, 1024, 64, sink)
    assert ms > 0 and nbytes == 1024 * 4 * 64 * 8 * 1024
    assert 1e3 < nbytes / ms / 1e6 < 45e3            # GB/s: above one CU's share, below the 39.3 TB/s of the return path + slack
    ms, flops = sptir.sptir_roof_fma(2048, 1024, sink)
    assert ms > 0 and 5.0 < flops / ms / 1e9 < 320.0  # TFLOP/s
    assert float(sink.sum()) == 0.0
    for bad in ((X, 0, 4, 8, 8), (X, 4096, 9, 8, 8), (X, 4096, 4, 0, 8), (X, 4096, 4, 8, 0)):
        with pytest.raises(sptir.SptirError):
            sptir.sptir_roof_gather(*bad, sink)


def test_build_options_are_validated(gpu_lib):
    w = ragged_workload(1, 50, 60, 4, max_deg=20)
    d = upload(w)
    for bad in ({"row_block": 48}, {"row_block": 512}, {"rounds": 3}, {"heavy_len": -1}, {"parts_per_launch": -2}):
        with pytest.raises(gpu_lib.SptirError) as e:
            gpu_lib.sptir_hyb_build_ex(w.n_rows, w.n_cols, d.indptr, d.indices, d.values, 2, 2, bad)
        assert e.value.status == 1, bad
    with pytest.raises(KeyError):
        gpu_lib.sptir_hyb_build_ex(w.n_rows, w.n_cols, d.indptr, d.indices, d.values, 2, 2, {"no_such_field": 1})


@pytest.mark.parametrize("feat", [128, 256, 320, 384, 520])
def test_spmm_feature_sweeps(gpu_lib, feat):
    """Where every launch reads back the Y of the one before it (no rounds), a Y too wide for the memory-side
    cache is produced in several sweeps over the launches, each over a group of 4 or 8 feature tiles; the limit
    is lowered here so that a small Y takes that path (feat = 320 and 520 have tile counts that do not split and
    run as one sweep)."""
    say(f"[feature sweeps] feat={feat}")
    w = ragged_workload(1300 + feat, 1500, 1800, feat, max_deg=900, long_rows=3)
    Yr, Sr = oracle.spmm_csr(w.n_rows, w.indptr, w.indices, w.values, w.X)
    d, hyb, got, want, info = build_both(gpu_lib, w, 3, 6, {"parts_per_launch": 1})
    assert info["n_phases"] == 3 and info["rounds"] == 0
    Y_one = torch.full((w.n_rows, feat), float("nan"), device="cuda")
    gpu_lib.sptir_spmm(hyb, d.X, Y_one)
    assert_y_close(Y_one.cpu().numpy(), Yr, Sr, what=f"one sweep feat={feat}")
    for limit_kb in (512, 1):   # 8 tiles of 1500 rows are 0.73 MB: sweeps of 4 tiles, then the same
        hyb2 = gpu_lib.sptir_hyb_build_ex(w.n_rows, w.n_cols, d.indptr, d.indices, d.values, 3, 6,
                                          {"parts_per_launch": 1, "sweep_kb": limit_kb})
        Y = torch.full((w.n_rows, feat), float("nan"), device="cuda")
        gpu_lib.sptir_spmm(hyb2, d.X, Y)
        assert torch.equal(Y, Y_one), f"feat={feat} limit={limit_kb} KB"
    # the same matrix in rounds, wider than one partial-sum row of the heavy pieces
    d, hyb3, got, want, info = build_both(gpu_lib, w, 3, 6, {"rounds": 1})
    assert info["rounds"] == 1 and info["n_heavy_pieces"] > 0
    Y = torch.full((w.n_rows, feat), float("nan"), device="cuda")
    gpu_lib.sptir_spmm(hyb3, d.X, Y)
    assert_y_close(Y.cpu().numpy(), Yr, Sr, what=f"rounds feat={feat}")
    # and with its X (1800 rows: 0.22 MB per tile) declared too wide for one sweep: groups of 8 or 4 tiles, the
    # heavy pieces of each group right after its lists; every sum is formed as before
    for limit_kb in (1900, 1):
        hyb4 = gpu_lib.sptir_hyb_build_ex(w.n_rows, w.n_cols, d.indptr, d.indices, d.values, 3, 6,
                                          {"rounds": 1, "sweep_kb": limit_kb})
        Y2 = torch.full((w.n_rows, feat), float("nan"), device="cuda")
        gpu_lib.sptir_spmm(hyb4, d.X, Y2)
        assert torch.equal(Y2, Y), f"rounds feat={feat} limit={limit_kb} KB"


@pytest.mark.parametrize("c", [1, 2, 4, 9])
def test_spmm_many_columns(gpu_lib, c):
    """More than 2^20 columns do not fit the 20-bit column field of the 8-byte stream records: 12-byte records."""
    n_rows, n_cols, feat = 700, 2_500_000, 4
    say(f"[many columns] c={c}")
    w = ragged_workload(900 + c, n_rows, n_cols, feat, max_deg=400, long_rows=4)
    d, hyb, got, want, info = build_both(gpu_lib, w, c, 5)
    assert_same_hyb(got, want)
    Y = torch.full((n_rows, feat), float("nan"), device="cuda")
    gpu_lib.sptir_spmm(hyb, d.X, Y)
    Yr, Sr = oracle.spmm_csr(w.n_rows, w.indptr, w.indices, w.values, w.X)
    assert_y_close(Y.cpu().numpy(), Yr, Sr, what=f"many columns c={c}")


@pytest.mark.parametrize("c,k,feat", [(1, 3, 32), (3, 5, 64), (2, 30, 8), (4, 11, 100), (1, 0, 3), (2, 4, 516)])
def test_spmm_long_rows(gpu_lib, c, k, feat):
    """Rows with far more non-zeros than a wavefront's list should hold (remainder pieces, and ELL rows when k is
    large) are heavy pieces: their chunks run through many heavy lists, whose partial sums (also of several
    heavy pieces of one row, c > 1, and of Y wider than one partial-sum row) land in the same row of Y."""
    say(f"[long rows] c={c} k={k} feat={feat}")
    w = ragged_workload(500 + c + k, 900, 40_000, feat, max_deg=30_000, long_rows=7)
    d, hyb, got, want, info = build_both(gpu_lib, w, c, k)
    assert_same_hyb(got, want)
    Yr, Sr = oracle.spmm_csr(w.n_rows, w.indptr, w.indices, w.values, w.X)
    Ys = []
    for _ in range(2):
        Y = torch.full((w.n_rows, feat), float("nan"), device="cuda")
        gpu_lib.sptir_spmm(hyb, d.X, Y)
        assert_y_close(Y.cpu().numpy(), Yr, Sr, what=f"long rows c={c} k={k}")
        Ys.append(Y)
    assert torch.equal(Ys[0], Ys[1])


def test_sweep_module_runs(gpu_lib, monkeypatch, capsys):
    """The c / d sweep driver runs end to end on the smallest graph and prints one JSON record per point."""
    import json
    from paper_2207_04606_amd import sweep
    monkeypatch.setattr("sys.argv", ["sweep", "--config", "tiny", "--reps", "1", "--c-values", "1,3", "--d-values", "8,33"])
    sweep.main()
    lines = [json.loads(l) for l in capsys.readouterr().out.splitlines() if l.startswith("{")]
    assert [(p["sweep"], p["c"], p["feat"]) for p in lines] == [("c", 1, 128), ("c", 3, 128), ("d", 1, 8), ("d", 1, 33)]
    assert all(p["hyb_ms"] > 0 and p["no_hyb_ms"] > 0 for p in lines)


def test_hyb_search_picks_a_candidate(gpu_lib):
    """The format search returns one of its candidates, built exactly like a direct build with that c."""
    w = ragged_workload(77, 3000, 3500, 64, max_deg=900, long_rows=6)
    d = upload(w)
    hyb, best_c, ms = gpu_lib.sptir_hyb_search(w.n_rows, w.n_cols, d.indptr, d.indices, d.values, 64,
                                               c_candidates=(1, 3, 8), max_bucket_log2=5, reps=2)
    assert best_c in (1, 3, 8) and len(ms) == 3 and all(t > 0 for t in ms)
    assert best_c == (1, 3, 8)[int(np.argmin(ms))]
    got, info = fetch_hyb(gpu_lib, hyb)
    assert info["n_col_parts"] == best_c and info["max_bucket_log2"] == 5
    assert_same_hyb(got, oracle.hyb_build(w.n_rows, w.n_cols, w.indptr, w.indices, w.values, best_c, 5))
    Y = torch.full((w.n_rows, 64), float("nan"), device="cuda")
    gpu_lib.sptir_spmm(hyb, d.X, Y)
    Yr, Sr = oracle.spmm_csr(w.n_rows, w.indptr, w.indices, w.values, w.X)
    assert_y_close(Y.cpu().numpy(), Yr, Sr, what="search")
    # defaults: the paper's candidate set and its rule for k
    hyb2, c2, _ = gpu_lib.sptir_hyb_search(w.n_rows, w.n_cols, d.indptr, d.indices, d.values, 32)
    info2 = gpu_lib.sptir_hyb_info(hyb2)
    assert c2 in (1, 2, 4, 8, 16) and info2["n_col_parts"] == c2
    assert info2["max_bucket_log2"] == gpu_lib.sptir_default_bucket_log2(w.nnz, w.n_rows)
    with pytest.raises(gpu_lib.SptirError):
        gpu_lib.sptir_hyb_search(w.n_rows, w.n_cols, d.indptr, d.indices, d.values, 32, c_candidates=(2, 0))


@pytest.mark.parametrize("name,feat", [("small", 32), ("small", 128), ("medium", 64), ("medium", 256)])
def test_launch_plan_query_matches_what_is_built(gpu_lib, name, feat):
    """The host-only query announces the row blocks and launches that a search at the same feature size builds."""
    w = workloads.make_config(name)
    d = upload(w)
    hyb, _, _ = gpu_lib.sptir_hyb_search(w.n_rows, w.n_cols, d.indptr, d.indices, d.values, feat,
                                         c_candidates=(w.n_col_parts,), max_bucket_log2=w.max_bucket_log2, reps=1)
    info = gpu_lib.sptir_hyb_info(hyb)
    plan = gpu_lib.sptir_launch_plan(w.n_rows, w.n_cols, info["n_ell_slots"] + info["n_rem_nnz"], w.n_col_parts, feat)
    assert (plan["row_block"], plan["n_launches"], plan["rounds"]) == (info["row_block"], info["n_phases"], info["rounds"])


def test_spmm_and_sddmm_replay_in_a_hip_graph(gpu_lib):
    """sptir_spmm / sptir_sddmm only enqueue kernels, so a stream capture records them; every replay (with
    eager work and synchronisation in between, and new operand values) must match the eager result."""
    w = workloads.make_config("small")
    d, hyb, got, want, info = build_both(gpu_lib, w, w.n_col_parts, w.max_bucket_log2)
    plan = gpu_lib.sptir_sddmm_plan_build(w.n_rows, w.n_cols, d.indptr, d.indices, 8)
    X = d.X.clone()
    Xl = torch.randn(w.n_rows, w.feat, device="cuda")
    Y = torch.empty(w.n_rows, w.feat, device="cuda")
    B = torch.empty(w.nnz, device="cuda")
    gpu_lib.sptir_spmm(hyb, X, Y)                      # first calls outside the capture (one-time set-up)
    gpu_lib.sptir_sddmm(plan, d.values, Xl, X, B)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            gpu_lib.sptir_spmm(hyb, X, Y, stream=side)
            gpu_lib.sptir_sddmm(plan, d.values, Xl, X, B, stream=side)
    torch.cuda.synchronize()
    for rep in range(3):
        X.copy_(torch.randn_like(X))                   # new values in the captured buffers
        Y.fill_(float("nan")); B.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        Y_eager = torch.empty_like(Y); B_eager = torch.empty_like(B)
        gpu_lib.sptir_spmm(hyb, X, Y_eager)
        gpu_lib.sptir_sddmm(plan, d.values, Xl, X, B_eager)
        torch.cuda.synchronize()
        assert torch.equal(Y, Y_eager) and torch.equal(B, B_eager), f"replay {rep}"
