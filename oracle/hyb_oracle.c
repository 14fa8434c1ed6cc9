/*
 * CPU oracle for hyb(c,k) construction and SpMM.  TEST INFRASTRUCTURE ONLY:
 * it exists to check the GPU library and to be timed as a CPU baseline; the
 * product path never calls it, and it shares no source with the GPU code.
 *
 * What it follows:
 *  - SpMM is the definition Y[i,k] = sum_j A[i,j] * X[j,k] (the SpMM equation
 *    of Section 4.2.1), with the result initialised to zero before the sum
 *    (the init block of the SpMM script in Appendix A), so empty rows give 0.
 *    Inputs are fp32; every product and sum is carried out in fp64, terms in
 *    CSR order.
 *  - hyb(c,k) follows Section 4.2.1: columns are cut into c partitions of
 *    width w; inside a partition a row piece of length l with
 *    2^(i-1) < l <= 2^i goes to bucket i and is padded to 2^i; each bucket is
 *    an ELL matrix.  The figure of hyb(2,2) shows k+1 = 3 buckets per
 *    partition, i.e. i = 0..k.  ELL storage is row-major (the flattening rule
 *    of Section 3.4.1 applied to the ELL axes of Appendix A).
 *  Readings where the paper is silent (all mirrored by the GPU library):
 *  - w = ceil(n_cols / c); the last partition may be narrower or empty.
 *  - a piece longer than 2^k is kept, unpadded, in a CSR remainder of its
 *    partition;
 *  - rows appear in a bucket in ascending row order, entries in CSR order;
 *  - a pad slot holds value +0.0f and repeats the last real column of its row
 *    piece; column ids are global;
 *  - empty buckets are kept (zero rows) so bucket id = p*(k+1)+i.
 *
 * The construction below is a literal two-pass "count, then append in order"
 * over (partition, row); nothing is blocked, fused or reordered.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
  int32_t n_rows, n_cols, c, k, w;
  int64_t n_buckets;        /* B = c*(k+1) */
  int64_t n_ell_rows;       /* R */
  int64_t n_slots;          /* S, pads included */
  int64_t n_rem_segs;       /* M */
  int64_t n_rem_nnz;        /* T */
  int64_t* bucket_row_ptr;  /* [B+1] */
  int64_t* bucket_slot_ptr; /* [B+1] */
  int32_t* ell_row;         /* [R] */
  int32_t* ell_col;         /* [S] */
  float*   ell_val;         /* [S] */
  int32_t* rem_part_ptr;    /* [c+1] */
  int32_t* rem_row;         /* [M] */
  int64_t* rem_ptr;         /* [M+1] */
  int32_t* rem_col;         /* [T] */
  float*   rem_val;         /* [T] */
} oracle_hyb_t;

/* smallest i with l <= 2^i, for l >= 1 (so 1->0, 2->1, 3..4->2, 5..8->3 ...) */
static int bucket_of_length(int64_t l) {
  int i = 0;
  while (((int64_t)1 << i) < l) ++i;
  return i;
}

/* first position q in [lo,hi) with indices[q] >= bound (columns ascend) */
static int64_t first_not_less(const int32_t* indices, int64_t lo, int64_t hi, int64_t bound) {
  int64_t q = lo;
  while (q < hi && (int64_t)indices[q] < bound) ++q;
  return q;
}

void oracle_hyb_free(oracle_hyb_t* h) {
  if (!h) return;
  free(h->bucket_row_ptr); free(h->bucket_slot_ptr); free(h->ell_row); free(h->ell_col);
  free(h->ell_val); free(h->rem_part_ptr); free(h->rem_row); free(h->rem_ptr);
  free(h->rem_col); free(h->rem_val);
  memset(h, 0, sizeof(*h));
}

/* returns 0 ok, 1 invalid argument, 2 columns not strictly ascending / out of range, 4 no memory */
int oracle_hyb_build(int32_t n_rows, int32_t n_cols, const int32_t* indptr, const int32_t* indices,
                     const float* values, int32_t c, int32_t k, oracle_hyb_t* h) {
  memset(h, 0, sizeof(*h));
  if (n_rows < 0 || n_cols < 0 || c < 1 || k < 0 || k > 30) return 1;
  if (indptr[0] != 0) return 1;
  for (int32_t r = 0; r < n_rows; ++r) {
    if (indptr[r + 1] < indptr[r]) return 1;
    for (int64_t q = indptr[r]; q < indptr[r + 1]; ++q) {
      if (indices[q] < 0 || indices[q] >= n_cols) return 2;
      if (q > indptr[r] && indices[q] <= indices[q - 1]) return 2;
    }
  }
  int32_t w = (int32_t)(((int64_t)n_cols + c - 1) / c);
  int64_t B = (int64_t)c * (k + 1);
  h->n_rows = n_rows; h->n_cols = n_cols; h->c = c; h->k = k; h->w = w; h->n_buckets = B;

  /* pass 1: how many rows land in each bucket, how much goes to each remainder */
  int64_t* rows_in = (int64_t*)calloc((size_t)B + 1, sizeof(int64_t));
  int64_t* rem_segs = (int64_t*)calloc((size_t)c + 1, sizeof(int64_t));
  int64_t* rem_nnz = (int64_t*)calloc((size_t)c + 1, sizeof(int64_t));
  if (!rows_in || !rem_segs || !rem_nnz) return 4;
  for (int32_t p = 0; p < c; ++p) {
    int64_t col_lo = (int64_t)p * w, col_hi = (int64_t)(p + 1) * w;
    for (int32_t r = 0; r < n_rows; ++r) {
      int64_t a = first_not_less(indices, indptr[r], indptr[r + 1], col_lo);
      int64_t b = first_not_less(indices, a, indptr[r + 1], col_hi);
      int64_t l = b - a;
      if (l == 0) continue;
      int i = bucket_of_length(l);
      if (i <= k) rows_in[(int64_t)p * (k + 1) + i] += 1;
      else { rem_segs[p] += 1; rem_nnz[p] += l; }
    }
  }
  h->bucket_row_ptr = (int64_t*)calloc((size_t)B + 1, sizeof(int64_t));
  h->bucket_slot_ptr = (int64_t*)calloc((size_t)B + 1, sizeof(int64_t));
  h->rem_part_ptr = (int32_t*)calloc((size_t)c + 1, sizeof(int32_t));
  if (!h->bucket_row_ptr || !h->bucket_slot_ptr || !h->rem_part_ptr) return 4;
  for (int64_t b = 0; b < B; ++b) {
    int i = (int)(b % (k + 1));
    h->bucket_row_ptr[b + 1] = h->bucket_row_ptr[b] + rows_in[b];
    h->bucket_slot_ptr[b + 1] = h->bucket_slot_ptr[b] + rows_in[b] * ((int64_t)1 << i);
  }
  int64_t M = 0, T = 0;
  for (int32_t p = 0; p < c; ++p) {
    M += rem_segs[p]; T += rem_nnz[p];
    if (M > INT32_MAX) return 1;
    h->rem_part_ptr[p + 1] = (int32_t)M;
  }
  h->n_ell_rows = h->bucket_row_ptr[B]; h->n_slots = h->bucket_slot_ptr[B];
  h->n_rem_segs = M; h->n_rem_nnz = T;
  h->ell_row = (int32_t*)malloc(sizeof(int32_t) * (size_t)(h->n_ell_rows + 1));
  h->ell_col = (int32_t*)malloc(sizeof(int32_t) * (size_t)(h->n_slots + 1));
  h->ell_val = (float*)malloc(sizeof(float) * (size_t)(h->n_slots + 1));
  h->rem_row = (int32_t*)malloc(sizeof(int32_t) * (size_t)(M + 1));
  h->rem_ptr = (int64_t*)calloc((size_t)M + 1, sizeof(int64_t));
  h->rem_col = (int32_t*)malloc(sizeof(int32_t) * (size_t)(T + 1));
  h->rem_val = (float*)malloc(sizeof(float) * (size_t)(T + 1));
  if (!h->ell_row || !h->ell_col || !h->ell_val || !h->rem_row || !h->rem_ptr || !h->rem_col || !h->rem_val)
    return 4;

  /* pass 2: append, partition by partition, rows ascending */
  int64_t* next_row = (int64_t*)calloc((size_t)B + 1, sizeof(int64_t)); /* rows already placed per bucket */
  if (!next_row) return 4;
  int64_t m = 0, t = 0;
  for (int32_t p = 0; p < c; ++p) {
    int64_t col_lo = (int64_t)p * w, col_hi = (int64_t)(p + 1) * w;
    for (int32_t r = 0; r < n_rows; ++r) {
      int64_t a = first_not_less(indices, indptr[r], indptr[r + 1], col_lo);
      int64_t b = first_not_less(indices, a, indptr[r + 1], col_hi);
      int64_t l = b - a;
      if (l == 0) continue;
      int i = bucket_of_length(l);
      if (i <= k) {
        int64_t bk = (int64_t)p * (k + 1) + i;
        int64_t width = (int64_t)1 << i;
        int64_t q = next_row[bk]++;
        h->ell_row[h->bucket_row_ptr[bk] + q] = r;
        int64_t base = h->bucket_slot_ptr[bk] + q * width;
        for (int64_t j = 0; j < l; ++j) {
          h->ell_col[base + j] = indices[a + j];
          h->ell_val[base + j] = values[a + j];
        }
        for (int64_t j = l; j < width; ++j) {
          h->ell_col[base + j] = indices[b - 1];
          h->ell_val[base + j] = 0.0f;
        }
      } else {
        h->rem_row[m] = r;
        h->rem_ptr[m] = t;
        for (int64_t j = 0; j < l; ++j) {
          h->rem_col[t + j] = indices[a + j];
          h->rem_val[t + j] = values[a + j];
        }
        t += l; ++m;
      }
    }
  }
  h->rem_ptr[M] = T;
  free(rows_in); free(rem_segs); free(rem_nnz); free(next_row);
  return 0;
}

/*
 * SpMM by definition on the CSR input.  Y [n_rows, feat] and (optionally) the
 * magnitude sum Sabs[i,k] = sum_j |A[i,j] * X[j,k]| used to normalise errors.
 * Rows are independent, so the row loop may be split over threads; the sum
 * inside a row is always sequential in CSR order.
 */
void oracle_spmm_csr(int32_t n_rows, const int32_t* indptr, const int32_t* indices,
                     const float* values, const float* X, int32_t feat, double* Y, double* Sabs) {
#pragma omp parallel for schedule(dynamic, 64)
  for (int32_t i = 0; i < n_rows; ++i) {
    double* y = Y + (int64_t)i * feat;
    double* s = Sabs ? Sabs + (int64_t)i * feat : 0;
    for (int32_t f = 0; f < feat; ++f) { y[f] = 0.0; if (s) s[f] = 0.0; }
    for (int64_t q = indptr[i]; q < indptr[i + 1]; ++q) {
      double a = (double)values[q];
      const float* x = X + (int64_t)indices[q] * feat;
      for (int32_t f = 0; f < feat; ++f) {
        double prod = a * (double)x[f];
        y[f] += prod;
        if (s) s[f] += fabs(prod);
      }
    }
  }
}

/* Same definition for a chosen list of rows only: Y and Sabs are [n_sel, feat]. */
void oracle_spmm_csr_rows(int64_t n_sel, const int32_t* rows, const int32_t* indptr,
                          const int32_t* indices, const float* values, const float* X,
                          int32_t feat, double* Y, double* Sabs) {
#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t u = 0; u < n_sel; ++u) {
    int32_t i = rows[u];
    double* y = Y + u * feat;
    double* s = Sabs ? Sabs + u * feat : 0;
    for (int32_t f = 0; f < feat; ++f) { y[f] = 0.0; if (s) s[f] = 0.0; }
    for (int64_t q = indptr[i]; q < indptr[i + 1]; ++q) {
      double a = (double)values[q];
      const float* x = X + (int64_t)indices[q] * feat;
      for (int32_t f = 0; f < feat; ++f) {
        double prod = a * (double)x[f];
        y[f] += prod;
        if (s) s[f] += fabs(prod);
      }
    }
  }
}

/*
 * SpMM evaluated from the hyb arrays (pads included), sequentially: Y starts
 * at zero, every ELL sub-matrix and then every remainder piece adds its
 * contribution.  Used to tie the format half of the oracle to the SpMM half.
 */
void oracle_spmm_hyb(const oracle_hyb_t* h, const float* X, int32_t feat, double* Y) {
  for (int64_t e = 0; e < (int64_t)h->n_rows * feat; ++e) Y[e] = 0.0;
  for (int64_t b = 0; b < h->n_buckets; ++b) {
    int64_t width = (int64_t)1 << (int)(b % (h->k + 1));
    int64_t nrow = h->bucket_row_ptr[b + 1] - h->bucket_row_ptr[b];
    for (int64_t q = 0; q < nrow; ++q) {
      double* y = Y + (int64_t)h->ell_row[h->bucket_row_ptr[b] + q] * feat;
      for (int64_t j = 0; j < width; ++j) {
        int64_t s = h->bucket_slot_ptr[b] + q * width + j;
        double a = (double)h->ell_val[s];
        const float* x = X + (int64_t)h->ell_col[s] * feat;
        for (int32_t f = 0; f < feat; ++f) y[f] += a * (double)x[f];
      }
    }
  }
  for (int64_t m = 0; m < h->n_rem_segs; ++m) {
    double* y = Y + (int64_t)h->rem_row[m] * feat;
    for (int64_t s = h->rem_ptr[m]; s < h->rem_ptr[m + 1]; ++s) {
      double a = (double)h->rem_val[s];
      const float* x = X + (int64_t)h->rem_col[s] * feat;
      for (int32_t f = 0; f < feat; ++f) y[f] += a * (double)x[f];
    }
  }
}

int oracle_num_threads(void) {
  int n = 1;
#ifdef _OPENMP
#pragma omp parallel
  {
#pragma omp single
    n = omp_get_num_threads();
  }
#endif
  return n;
}
