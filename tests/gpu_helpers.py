"""Helpers of the GPU parity tests: upload a workload, fetch the hyb arrays,
compare Y with the oracle under the normalised-error criterion."""
import types

import numpy as np
import torch

import hyb_checks

# max |Y_gpu - Y_oracle| / sum_j |a_ij x_jk|: fp32 products and sums against the
# fp64 oracle.  A row of n terms summed in fp32 in chunks errs by about
# u*sqrt(n) relative to the magnitude sum (u = 2^-24 = 6e-8), i.e. below 1e-5
# up to n ~ 2.7e4 > the largest degree used here (21,657).
Y_TOL = 1e-5


def upload(w):
    dev = torch.device("cuda:0")
    return types.SimpleNamespace(
        indptr=torch.from_numpy(w.indptr).to(dev), indices=torch.from_numpy(w.indices).to(dev),
        values=torch.from_numpy(w.values).to(dev), X=torch.from_numpy(w.X).to(dev))


def fetch_hyb(sptir, hyb):
    info = sptir.sptir_hyb_info(hyb)
    out = types.SimpleNamespace(n_rows=info["n_rows"], n_cols=info["n_cols"], c=info["n_col_parts"],
                                k=info["max_bucket_log2"], w=info["part_width"])
    for name in hyb_checks.ARRAY_NAMES:
        setattr(out, name, sptir.sptir_hyb_array(hyb, name))
    return out, info


def assert_y_close(Y_gpu, Y_ref, S_ref, tol=Y_TOL, what=""):
    Y_gpu = np.asarray(Y_gpu, dtype=np.float64)
    assert np.isfinite(Y_gpu).all(), f"{what}: non-finite output"
    err = np.abs(Y_gpu - Y_ref)
    zero = S_ref == 0
    assert (Y_gpu[zero] == 0).all(), f"{what}: entries with no contributing term must be exactly 0"
    ratio = err[~zero] / S_ref[~zero]
    worst = float(ratio.max()) if ratio.size else 0.0
    assert worst <= tol, f"{what}: max normalised error {worst:.3e} > {tol}"
    return worst
