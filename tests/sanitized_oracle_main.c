/*
 * Runs the C oracles and the column sampler as a stand-alone program, so that they can be built with
 * -fsanitize=address,undefined and fed the same inputs as the ordinary shared-library build
 * (tests/test_oracle_sanitized.py compares the two).  Test infrastructure only: it holds no arithmetic of
 * its own, it reads arrays from a file, calls the oracle and writes what came back.
 *
 *   prog hyb   in out    header int64[6] = n_rows n_cols nnz feat c k, then indptr i32[n_rows+1],
 *                        indices i32[nnz], values f32[nnz], X f32[n_cols*feat], X2 f32[n_rows*feat]
 *                        -> rc i64; if rc == 0: sizes i64[5] (B R S M T), the ten hyb arrays in the order of
 *                        the struct, Y_csr f64, Sabs f64, Y_hyb f64, Y_rows f64 (every second row),
 *                        sddmm B f64[nnz], M f64[nnz]
 *   prog rgms  in out    header int64[6] = n_rel n nnz d_in d_out 0, then indptr i32[n_rel*n+1], indices, values,
 *                        X f32[n*d_in], W f32[n_rel*d_in*d_out] -> Y f64[n*d_out], S f64[n*d_out]
 *   prog cols  in out    header int64[6] = n_rows n_cols nnz seed 0 0, then indptr i64[n_rows+1]
 *                        -> rc i64, indices i32[nnz]
 */
#include <stdio.h>
#include "../oracle/hyb_oracle.c"

void oracle_sddmm_csr(int32_t n_rows, const int32_t* indptr, const int32_t* indices, const float* values,
                      const float* X, const float* Yt, int32_t d, double* B_values, double* Mabs);
void oracle_rgms(int32_t n_rel, int32_t n_rows, const int32_t* indptr, const int32_t* indices, const float* values,
                 const float* X, const float* W, int32_t d_in, int32_t d_out, double* Y, double* Sabs);
int colsample_fill(int32_t n_rows, int32_t n_cols, const int64_t* indptr, uint64_t seed, int32_t* indices);

static void die(const char* what) { fprintf(stderr, "sanitized_oracle_main: %s\n", what); exit(3); }

/* exact-size heap blocks, so that the sanitizer sees an access one element past an array's end */
static void* room(size_t n, size_t size) {
  void* p = malloc(n * size ? n * size : 1);
  if (!p) die("out of memory");
  return p;
}
static void* get(FILE* f, size_t n, size_t size) {
  void* p = room(n, size);
  if (n && fread(p, size, n, f) != n) die("short input file");
  return p;
}
static void put(FILE* f, const void* p, size_t n, size_t size) {
  if (n && fwrite(p, size, n, f) != n) die("short write");
}

int main(int argc, char** argv) {
  if (argc != 4) die("usage: prog hyb|rgms|cols in out");
  FILE* in = fopen(argv[2], "rb");
  FILE* out = fopen(argv[3], "wb");
  if (!in || !out) die("cannot open files");
  int64_t hd[6];
  if (fread(hd, sizeof(int64_t), 6, in) != 6) die("no header");
  if (!strcmp(argv[1], "hyb")) {
    int32_t n_rows = (int32_t)hd[0], n_cols = (int32_t)hd[1], feat = (int32_t)hd[3];
    int64_t nnz = hd[2];
    int32_t* indptr = get(in, (size_t)n_rows + 1, 4);
    int32_t* indices = get(in, (size_t)nnz, 4);
    float* values = get(in, (size_t)nnz, 4);
    float* X = get(in, (size_t)n_cols * feat, 4);
    float* X2 = get(in, (size_t)n_rows * feat, 4);
    oracle_hyb_t h;
    memset(&h, 0, sizeof(h));
    int64_t rc = oracle_hyb_build(n_rows, n_cols, indptr, indices, values, (int32_t)hd[4], (int32_t)hd[5], &h);
    put(out, &rc, 1, 8);
    if (rc == 0) {
      int64_t sizes[5] = {h.n_buckets, h.n_ell_rows, h.n_slots, h.n_rem_segs, h.n_rem_nnz};
      put(out, sizes, 5, 8);
      put(out, h.bucket_row_ptr, (size_t)h.n_buckets + 1, 8);
      put(out, h.bucket_slot_ptr, (size_t)h.n_buckets + 1, 8);
      put(out, h.ell_row, (size_t)h.n_ell_rows, 4);
      put(out, h.ell_col, (size_t)h.n_slots, 4);
      put(out, h.ell_val, (size_t)h.n_slots, 4);
      put(out, h.rem_part_ptr, (size_t)h.c + 1, 4);
      put(out, h.rem_row, (size_t)h.n_rem_segs, 4);
      put(out, h.rem_ptr, (size_t)h.n_rem_segs + 1, 8);
      put(out, h.rem_col, (size_t)h.n_rem_nnz, 4);
      put(out, h.rem_val, (size_t)h.n_rem_nnz, 4);
      size_t ny = (size_t)n_rows * feat;
      double* Y = room(ny, 8);
      double* S = room(ny, 8);
      oracle_spmm_csr(n_rows, indptr, indices, values, X, feat, Y, S);
      put(out, Y, ny, 8);
      put(out, S, ny, 8);
      oracle_spmm_hyb(&h, X, feat, Y);
      put(out, Y, ny, 8);
      int64_t n_sel = (n_rows + 1) / 2;
      int32_t* rows = room((size_t)n_sel, 4);
      for (int64_t u = 0; u < n_sel; ++u) rows[u] = (int32_t)(2 * u);
      oracle_spmm_csr_rows(n_sel, rows, indptr, indices, values, X, feat, Y, S);
      put(out, Y, (size_t)n_sel * feat, 8);
      double* B = room((size_t)nnz, 8);
      double* M = room((size_t)nnz, 8);
      oracle_sddmm_csr(n_rows, indptr, indices, values, X2, X, feat, B, M);
      put(out, B, (size_t)nnz, 8);
      put(out, M, (size_t)nnz, 8);
      free(Y); free(S); free(rows); free(B); free(M);
    }
    oracle_hyb_free(&h);
    free(indptr); free(indices); free(values); free(X); free(X2);
  } else if (!strcmp(argv[1], "rgms")) {
    int32_t n_rel = (int32_t)hd[0], n = (int32_t)hd[1], d_in = (int32_t)hd[3], d_out = (int32_t)hd[4];
    int64_t nnz = hd[2];
    int32_t* indptr = get(in, (size_t)n_rel * n + 1, 4);
    int32_t* indices = get(in, (size_t)nnz, 4);
    float* values = get(in, (size_t)nnz, 4);
    float* X = get(in, (size_t)n * d_in, 4);
    float* W = get(in, (size_t)n_rel * d_in * d_out, 4);
    size_t ny = (size_t)n * d_out;
    double* Y = room(ny, 8);
    double* S = room(ny, 8);
    oracle_rgms(n_rel, n, indptr, indices, values, X, W, d_in, d_out, Y, S);
    put(out, Y, ny, 8);
    put(out, S, ny, 8);
    free(indptr); free(indices); free(values); free(X); free(W); free(Y); free(S);
  } else if (!strcmp(argv[1], "cols")) {
    int32_t n_rows = (int32_t)hd[0], n_cols = (int32_t)hd[1];
    int64_t nnz = hd[2];
    int64_t* indptr = get(in, (size_t)n_rows + 1, 8);
    int32_t* indices = room((size_t)nnz, 4);
    int64_t rc = colsample_fill(n_rows, n_cols, indptr, (uint64_t)hd[3], indices);
    put(out, &rc, 1, 8);
    if (rc == 0) put(out, indices, (size_t)nnz, 4);
    free(indptr); free(indices);
  } else {
    die("unknown mode");
  }
  fclose(in);
  if (fclose(out) != 0) die("close failed");
  return 0;
}
