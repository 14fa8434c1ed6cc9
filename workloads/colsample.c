/*
 * Seeded column sampler for synthetic graphs (input generation only).
 *
 * For every row r it draws deg[r] distinct column ids uniformly from
 * [0, n_cols) and stores them in ascending order at indices[indptr[r] ...].
 * The random stream of a row depends only on (seed, r), so the output is
 * the same for any thread count.  This file holds no SpMM or hyb logic: it
 * only manufactures the CSR column structure that both the CPU oracle and
 * the GPU library are later fed with.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static inline uint64_t mix64(uint64_t z) {
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

typedef struct { uint64_t key, ctr; } rng_t;

static inline uint64_t rng_next(rng_t* g) { return mix64(g->key ^ mix64(g->ctr++)); }

/* unbiased integer in [0, n) by rejection on the top multiple of n */
static inline uint32_t rng_below(rng_t* g, uint32_t n) {
  uint64_t lim = (0xFFFFFFFFFFFFFFFFull / n) * n;
  uint64_t x;
  do { x = rng_next(g); } while (x >= lim);
  return (uint32_t)(x % n);
}

static int cmp_i32(const void* a, const void* b) {
  int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
  return (x > y) - (x < y);
}

/* returns 0 on success, 1 on bad arguments, 2 on allocation failure */
int colsample_fill(int32_t n_rows, int32_t n_cols, const int64_t* indptr,
                   uint64_t seed, int32_t* indices) {
  if (n_rows < 0 || n_cols <= 0) return 1;
  for (int32_t r = 0; r < n_rows; ++r) {
    int64_t d = indptr[r + 1] - indptr[r];
    if (d < 0 || d > n_cols) return 1;
  }
  int fail = 0;
  size_t words = ((size_t)n_cols + 63) / 64;
#pragma omp parallel
  {
    uint64_t* bits = (uint64_t*)calloc(words, sizeof(uint64_t));
    if (!bits) {
#pragma omp atomic write
      fail = 2;
    }
#pragma omp barrier
    if (!fail) {
#pragma omp for schedule(dynamic, 64)
      for (int32_t r = 0; r < n_rows; ++r) {
        int64_t d = indptr[r + 1] - indptr[r];
        int32_t* out = indices + indptr[r];
        if (d == 0) continue;
        rng_t g = { mix64(seed ^ 0xC01C01C01ull) ^ mix64((uint64_t)r * 0xD1342543DE82EF95ull + 1), 0 };
        /* draw the smaller of the set and its complement */
        int complement = (d > n_cols / 2);
        int64_t m = complement ? (int64_t)n_cols - d : d;
        int64_t got = 0;
        while (got < m) {
          uint32_t c = rng_below(&g, (uint32_t)n_cols);
          uint64_t bit = 1ull << (c & 63);
          if (bits[c >> 6] & bit) continue;
          bits[c >> 6] |= bit;
          if (!complement) out[got] = (int32_t)c;
          ++got;
        }
        if (!complement && (size_t)d * 24 < (size_t)n_cols) {
          /* sparse row: sort the drawn list, then clear its bits */
          for (int64_t j = 0; j < d; ++j) bits[out[j] >> 6] = 0;
          qsort(out, (size_t)d, sizeof(int32_t), cmp_i32);
        } else {
          /* dense row: read the members (or non-members) off the bitmap */
          int64_t j = 0;
          for (size_t wd = 0; wd < words; ++wd) {
            uint64_t v = complement ? ~bits[wd] : bits[wd];
            bits[wd] = 0;
            while (v) {
              int b = __builtin_ctzll(v);
              v &= v - 1;
              int64_t c = (int64_t)wd * 64 + b;
              if (c < n_cols) out[j++] = (int32_t)c;
            }
          }
        }
      }
    }
    free(bits);
  }
  return fail;
}
