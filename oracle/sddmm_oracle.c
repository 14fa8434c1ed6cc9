/*
 * CPU oracle for SDDMM.  TEST INFRASTRUCTURE ONLY: it exists to check the GPU
 * library and to be timed as a CPU baseline; the product path never calls it,
 * and it shares no source with the GPU code.
 *
 * What it follows: the SDDMM equation of the SDDMM subsection of Section 4.2,
 *     B[i,j] = sum_{k=1..d} A[i,j] * X[i,k] * Y[k,j]   for the stored (i,j) of A,
 * where A and B share one sparse structure (CSR here, as for SpMM), X is
 * n_rows x d and Y is d x n_cols.  Inputs are fp32; every product and sum is
 * carried out in fp64, k ascending.
 *  Reading where the paper is silent: the memory layout of Y.  The equation
 *  reads column j of Y for entry (i,j); here the caller hands over the
 *  transpose Yt (n_cols x d, row-major), so that column is one contiguous row,
 *  the same layout as X.  Yt[j,k] == Y[k,j].
 *  The result array is parallel to A's values: B_values[q] belongs to the same
 *  (row, column) as values[q].
 *
 * Also returns, per entry, M[q] = |A[i,j]| * sum_k |X[i,k] * Y[k,j]|, the
 * magnitude sum against which a float32 result's error is normalised.
 */
#include <stdint.h>
#include <math.h>

void oracle_sddmm_csr(int32_t n_rows, const int32_t* indptr, const int32_t* indices, const float* values,
                      const float* X, const float* Yt, int32_t d, double* B_values, double* Mabs) {
#pragma omp parallel for schedule(dynamic, 64)
  for (int32_t i = 0; i < n_rows; ++i) {
    const float* x = X + (int64_t)i * d;
    for (int64_t q = indptr[i]; q < indptr[i + 1]; ++q) {
      const float* y = Yt + (int64_t)indices[q] * d;
      double a = (double)values[q];
      double sum = 0.0, mag = 0.0;
      for (int32_t k = 0; k < d; ++k) {
        double term = a * (double)x[k] * (double)y[k];
        sum += term;
        mag += fabs(term);
      }
      B_values[q] = sum;
      if (Mabs) Mabs[q] = mag;
    }
  }
}
