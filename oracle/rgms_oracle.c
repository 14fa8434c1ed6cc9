/*
 * CPU oracle for the relational gather-matmul-scatter operator (RGMS).  TEST
 * INFRASTRUCTURE ONLY: it exists to check the GPU library and to be timed as
 * a CPU baseline; the product path never calls it and shares no source with it.
 *
 * What it follows: the RGMS equation of the RGMS subsection (Section 4.4),
 *     Y[i,l] = sum_{r=1..R} sum_{j=1..n} sum_{k=1..d_in} A[r,i,j] * X[j,k] * W[r,k,l],
 * with A a 3-D sparse tensor whose slice r is the 2-D sparse matrix of
 * relation r, X dense n_cols x d_in, W dense R x d_in x d_out.  Inputs are
 * fp32; every product and sum is carried out in fp64, in the order of the
 * three sums of the equation (r, then j in CSR order, then k).
 *  Readings where the paper is silent:
 *  - A is stored slice after slice in CSR: indptr has R*n_rows + 1 entries,
 *    "stacked row" r*n_rows + i holds the entries A[r,i,:] (the dense-fixed R
 *    and I axes followed by a sparse-variable J axis, the way Appendix A
 *    declares axes);
 *  - W[r] is row-major d_in x d_out; Y is overwritten (rows without entries
 *    in any relation become 0), as for SpMM.
 * Also returns S[i,l] = sum |A[r,i,j] * X[j,k] * W[r,k,l]|, the magnitude
 * sum against which a float32 result's error is normalised.
 */
#include <stdint.h>
#include <math.h>

void oracle_rgms(int32_t n_rel, int32_t n_rows, const int32_t* indptr, const int32_t* indices, const float* values,
                 const float* X, const float* W, int32_t d_in, int32_t d_out, double* Y, double* Sabs) {
#pragma omp parallel for schedule(dynamic, 64)
  for (int32_t i = 0; i < n_rows; ++i) {
    double* y = Y + (int64_t)i * d_out;
    double* s = Sabs ? Sabs + (int64_t)i * d_out : 0;
    for (int32_t l = 0; l < d_out; ++l) { y[l] = 0.0; if (s) s[l] = 0.0; }
    for (int32_t r = 0; r < n_rel; ++r) {
      const float* w = W + (int64_t)r * d_in * d_out;
      int64_t row = (int64_t)r * n_rows + i;
      for (int64_t q = indptr[row]; q < indptr[row + 1]; ++q) {
        double a = (double)values[q];
        const float* x = X + (int64_t)indices[q] * d_in;
        for (int32_t k = 0; k < d_in; ++k) {
          double ax = a * (double)x[k];
          for (int32_t l = 0; l < d_out; ++l) {
            double term = ax * (double)w[(int64_t)k * d_out + l];
            y[l] += term;
            if (s) s[l] += fabs(term);
          }
        }
      }
    }
  }
}
