"""fp64 CPU oracle for hyb(c,k) construction, SpMM, SDDMM and RGMS.

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and
by bench.py's cpu_baseline leg.  The GPU product path never touches it.
"""
from .cpu import (HybArrays, build, hyb_build, num_threads, rgms, sddmm_csr, spmm_csr,
                  spmm_csr_rows, spmm_hyb)
