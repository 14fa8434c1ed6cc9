"""Seeded synthetic heterogeneous graphs for the relational gather-matmul-scatter
operator: a 3-D sparse tensor A[r, i, j] stored slice after slice in CSR
("stacked rows" r * n + i), a feature matrix X and one weight matrix per
relation.  The five configurations take the node, edge and edge-type counts
of the heterogeneous graphs in the paper's RGCN table; the graphs themselves
are synthetic.  No arithmetic of the operator lives here.

Recipe (numpy PCG64, one seed):
  * the E edges are dealt to the R relations with Zipf-like shares
    share_r ~ 1 / (1 + rank_r)^0.8 (every relation gets at least one edge);
  * inside a relation, destination rows follow a popularity law
    p_i ~ 1 / (1 + rank_i)^0.6 under a random ranking of the nodes, source
    columns are uniform; duplicate (r, i, j) triples are dropped;
  * values are 1 / (number of entries of (r, i)), the per-relation mean
    normalisation of relational graph convolution;
  * X ~ N(0, 1), W ~ N(0, 1 / d_in), float32.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

HETERO_CONFIGS = {
    "hetero_tiny": dict(n=300, edges=2000, n_rel=5),
    "hetero_a": dict(n=7262, edges=48810, n_rel=45),
    "hetero_b": dict(n=27163, edges=148100, n_rel=46),
    "hetero_c": dict(n=94806, edges=672884, n_rel=96),
    "hetero_d": dict(n=93773, edges=4762678, n_rel=51),
    "hetero_e": dict(n=1885136, edges=5668682, n_rel=96),
}


@dataclass
class HeteroWorkload:
    name: str
    n: int                  # nodes: A[r] is n x n
    n_rel: int
    indptr: np.ndarray      # int32 [n_rel * n + 1], stacked rows r * n + i
    indices: np.ndarray     # int32 [nnz], strictly ascending inside a stacked row
    values: np.ndarray      # float32 [nnz]
    X: np.ndarray           # float32 [n, d_in]
    W: np.ndarray           # float32 [n_rel, d_in, d_out]
    meta: dict = field(default_factory=dict)

    @property
    def nnz(self) -> int:
        return int(self.indices.shape[0])


def make_hetero(name: str, seed: int = 0, d_in: int = 32, d_out: int = 32, scale: float = 1.0) -> HeteroWorkload:
    cfg = HETERO_CONFIGS[name]
    n = max(4, int(round(cfg["n"] * scale)))
    n_rel = int(cfg["n_rel"])
    edges = max(n_rel, int(round(cfg["edges"] * scale)))
    rng = np.random.Generator(np.random.PCG64(seed))
    share = 1.0 / (1.0 + rng.permutation(n_rel)) ** 0.8
    per_rel = np.maximum(1, np.floor(share / share.sum() * edges)).astype(np.int64)
    popularity = 1.0 / (1.0 + rng.permutation(n)) ** 0.6
    cdf = np.cumsum(popularity)
    cdf /= cdf[-1]
    rel = np.repeat(np.arange(n_rel, dtype=np.int64), per_rel)
    rows = np.minimum(np.searchsorted(cdf, rng.random(rel.shape[0])), n - 1).astype(np.int64)
    cols = rng.integers(0, n, rel.shape[0], dtype=np.int64)
    key = np.unique((rel * n + rows) * n + cols)          # sorted by (r, i, j), duplicates dropped
    stacked = key // n
    indices = (key % n).astype(np.int32)
    counts = np.bincount(stacked, minlength=n_rel * n)
    if key.shape[0] >= 2**31:
        raise ValueError("nnz does not fit int32")
    indptr = np.zeros(n_rel * n + 1, dtype=np.int64)
    np.cumsum(counts, out=indptr[1:])
    values = (1.0 / counts[stacked]).astype(np.float32)
    X = rng.standard_normal((n, d_in), dtype=np.float32)
    W = (rng.standard_normal((n_rel, d_in, d_out), dtype=np.float32) / np.float32(np.sqrt(d_in))).astype(np.float32)
    return HeteroWorkload(name, n, n_rel, indptr.astype(np.int32), indices, values, X, W,
                          meta=dict(seed=seed, d_in=d_in, d_out=d_out, edges_target=edges,
                                    max_entries_per_stacked_row=int(counts.max())))
