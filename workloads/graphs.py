"""Seeded synthetic inputs shaped like the paper's GNN graphs (Table 1).

This module only manufactures inputs: CSR structure, fp32 values and the dense
feature matrix X.  It holds none of the hyb / SpMM arithmetic, and it is the
one piece of code the CPU oracle's tests and the GPU library's tests share.

The five named configurations take the node / edge counts of cora, pubmed,
ogbn-arxiv, ogbn-proteins and reddit (Table 1 of the paper); the structure is
synthetic (fitted power-law or clipped-normal out-degrees, columns uniform
without replacement) because the datasets themselves are not available.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "colsample.c")
_LIB = os.path.join(_HERE, "libcolsample.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the column sampler with gcc (host code only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.colsample_fill.restype = ctypes.c_int
        _lib.colsample_fill.argtypes = [
            ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p]
    return _lib


@dataclass
class Workload:
    name: str
    n_rows: int
    n_cols: int
    indptr: np.ndarray      # int32 [n_rows+1]
    indices: np.ndarray     # int32 [nnz], strictly ascending inside a row
    values: np.ndarray      # float32 [nnz]
    X: np.ndarray           # float32 [n_cols, feat], C order
    feat: int
    n_col_parts: int        # hyb parameter c of the configuration
    max_bucket_log2: int    # hyb parameter k of the configuration
    meta: dict = field(default_factory=dict)

    @property
    def nnz(self) -> int:
        return int(self.indices.shape[0])


def sample_columns(deg: np.ndarray, n_cols: int, seed: int):
    """deg[r] distinct sorted columns per row, uniform over [0, n_cols)."""
    deg = np.asarray(deg, dtype=np.int64)
    indptr = np.zeros(deg.shape[0] + 1, dtype=np.int64)
    np.cumsum(deg, out=indptr[1:])
    nnz = int(indptr[-1])
    if nnz >= 2**31:
        raise ValueError("nnz does not fit int32")
    indices = np.empty(nnz, dtype=np.int32)
    rc = _load().colsample_fill(
        deg.shape[0], n_cols, indptr.ctypes.data, seed, indices.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"colsample_fill failed with code {rc}")
    return indptr.astype(np.int32), indices


def power_law_degrees(n: int, nnz_target: int, alpha: float, dmax: int,
                      rng: np.random.Generator) -> np.ndarray:
    """deg_i = clip(floor(s * t_i), 1, dmax) with t_i Pareto(alpha-1) draws and
    the scale s fitted by bisection so that sum(deg) lands on nnz_target."""
    u = rng.random(n)
    t = (1.0 - u) ** (-1.0 / (alpha - 1.0))

    def total(s):
        return int(np.clip(np.floor(s * t), 1, dmax).sum())

    lo, hi = 0.0, 1.0
    while total(hi) < nnz_target and hi < 1e12:
        hi *= 2.0
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if total(mid) < nnz_target:
            lo = mid
        else:
            hi = mid
    return np.clip(np.floor(hi * t), 1, dmax).astype(np.int64)


def _uniform_pm1(rng, shape):
    return (rng.random(shape, dtype=np.float32) * np.float32(2.0) - np.float32(1.0))


def _uniform_01_closed(rng, n):
    return (np.float32(1.0) - rng.random(n, dtype=np.float32))


# name -> (n, nnz_target, feat, c, k, degree recipe, value recipe, X recipe)
CONFIGS = {
    "tiny": dict(n=2708, nnz=10556, feat=64, c=1, k=5, deg=("powerlaw", 2.1, None),
                 val="inv_deg_row", x="uniform"),
    "small": dict(n=19717, nnz=88651, feat=128, c=2, k=6, deg=("powerlaw", 2.2, None),
                  val="uniform01", x="uniform"),
    "medium": dict(n=169343, nnz=1166243, feat=128, c=4, k=9, deg=("powerlaw", 2.0, 13000),
                   val="sym_norm", x="normal"),
    "protein": dict(n=132534, nnz=39561252, feat=128, c=8, k=10, deg=("normal", 300.0, 100.0, 7750),
                    val="uniform01", x="normal"),
    "social": dict(n=232965, nnz=114615892, feat=256, c=16, k=11, deg=("powerlaw", 1.8, 21657),
                   val="inv_deg_row", x="normal"),
}
CONFIG_ORDER = ["tiny", "small", "medium", "protein", "social"]


def make_config(name: str, seed: int = 0, feat: int | None = None,
                scale: float = 1.0) -> Workload:
    """Build one of the five named workloads.  `scale` < 1 shrinks the node and
    edge counts proportionally (same recipe) for quick tests."""
    cfg = CONFIGS[name]
    n = max(4, int(round(cfg["n"] * scale)))
    nnz_target = max(n, int(round(cfg["nnz"] * scale)))
    feat = int(cfg["feat"] if feat is None else feat)
    rng = np.random.Generator(np.random.PCG64(seed))
    kind = cfg["deg"][0]
    if kind == "powerlaw":
        _, alpha, dmax = cfg["deg"]
        dmax = (n - 1) if dmax is None else min(int(dmax), n - 1)
        deg = power_law_degrees(n, nnz_target, alpha, dmax, rng)
    else:
        _, mu, sigma, dmax = cfg["deg"]
        mu_s = mu * (nnz_target / n) / (cfg["nnz"] / cfg["n"])
        deg = np.clip(np.rint(rng.normal(mu_s, sigma * mu_s / mu, n)), 1, min(dmax, n - 1)).astype(np.int64)
    indptr, indices = sample_columns(deg, n, seed)
    nnz = indices.shape[0]
    if cfg["val"] == "inv_deg_row":
        values = np.repeat((1.0 / deg).astype(np.float32), deg)
    elif cfg["val"] == "uniform01":
        values = _uniform_01_closed(rng, nnz)
    elif cfg["val"] == "sym_norm":
        di = np.repeat(deg.astype(np.float64), deg)
        dj = deg.astype(np.float64)[indices]
        values = (1.0 / np.sqrt(di * dj)).astype(np.float32)
    else:
        raise ValueError(cfg["val"])
    if cfg["x"] == "uniform":
        X = _uniform_pm1(rng, (n, feat))
    else:
        X = rng.standard_normal((n, feat), dtype=np.float32)
    meta = dict(config=name, seed=seed, scale=scale, nnz_target=nnz_target,
                max_degree=int(deg.max()), mean_degree=float(deg.mean()))
    return Workload(name, n, n, indptr, indices, values, np.ascontiguousarray(X), feat,
                    cfg["c"], cfg["k"], meta)


def random_csr(n_rows: int, n_cols: int, deg: np.ndarray, seed: int, feat: int,
               value_kind: str = "normal") -> Workload:
    """Free-form workload for tests: caller supplies the per-row lengths
    (zeros allowed), columns are uniform without replacement."""
    rng = np.random.Generator(np.random.PCG64(seed))
    deg = np.asarray(deg, dtype=np.int64)
    assert deg.shape[0] == n_rows and (deg <= n_cols).all() and (deg >= 0).all()
    indptr, indices = sample_columns(deg, n_cols, seed)
    nnz = indices.shape[0]
    if value_kind == "normal":
        values = rng.standard_normal(nnz, dtype=np.float32)
    elif value_kind == "ones":
        values = np.ones(nnz, dtype=np.float32)
    else:
        values = _uniform_01_closed(rng, nnz)
    X = rng.standard_normal((n_cols, feat), dtype=np.float32)
    return Workload("random", n_rows, n_cols, indptr, indices, values, X, feat, 1, 0,
                    dict(seed=seed))
