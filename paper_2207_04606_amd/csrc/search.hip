// Format search: the tuning rule of section 4.2.1 of arXiv 2207.04606, which
// tries c in {1, 2, 4, 8, 16} and sets k = ceil(log2(nnz / n)).  Here every
// candidate c is built and its SpMM is timed on scratch operands of the
// caller's feature size; the fastest decomposition is kept.
#include <vector>

#include "sptir_internal.h"

using namespace sptir;

extern "C" sptir_status_t sptir_hyb_search(const sptir_csr_t* csr, const int32_t* c_candidates, int32_t n_candidates,
                                           int32_t max_bucket_log2, int32_t feat, int32_t reps, void* stream_,
                                           sptir_hyb_t** out, int32_t* best_c, float* ms_per_candidate) {
  static const int32_t kPaperCandidates[] = {1, 2, 4, 8, 16};
  if (!csr || !out || feat < 1 || reps < 1 || n_candidates < 0) return SPTIR_ERR_INVALID_ARG;
  if (n_candidates > 0 && !c_candidates) return SPTIR_ERR_INVALID_ARG;
  if (n_candidates == 0) { c_candidates = kPaperCandidates; n_candidates = 5; }
  if (csr->n_rows < 0 || csr->n_cols < 0 || csr->nnz < 0) return SPTIR_ERR_INVALID_ARG;
  const int32_t k = max_bucket_log2 >= 0 ? max_bucket_log2 : sptir_default_bucket_log2(csr->nnz, csr->n_rows);
  hipStream_t stream = (hipStream_t)stream_;

  sptir_alloc_fn alloc; sptir_free_fn free_; void* actx;
  current_allocator(&alloc, &free_, &actx);
  const size_t x_bytes = sizeof(float) * (size_t)csr->n_cols * feat, y_bytes = sizeof(float) * (size_t)csr->n_rows * feat;
  float* X = (float*)alloc(x_bytes ? x_bytes : 16, actx, stream);
  float* Y = (float*)alloc(y_bytes ? y_bytes : 16, actx, stream);
  hipEvent_t e0 = nullptr, e1 = nullptr;
  sptir_hyb_t* best = nullptr;
  float best_ms = 0.f;
  int32_t best_candidate = 0;
  sptir_status_t st = SPTIR_OK;
  if (!X || !Y) { st = SPTIR_ERR_ALLOC; goto done; }
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) {
    st = note_hip_error(hipGetLastError(), "hipEventCreate"); goto done;
  }
  // the values of X do not change the time of a launch; zeros keep every product finite
  if (x_bytes && hipMemsetAsync(X, 0, x_bytes, stream) != hipSuccess) {
    st = note_hip_error(hipGetLastError(), "hipMemsetAsync"); goto done;
  }
  for (int32_t i = 0; i < n_candidates; ++i) {
    sptir_hyb_t* h = nullptr;
    sptir_build_options_t opt = complete_options(nullptr);
    opt.feat_hint = feat;  // launch plan sized for `feat`
    st = hyb_build_impl(csr, c_candidates[i], k, opt, stream_, &h);
    if (st != SPTIR_OK) goto done;
    float ms = 0.f;
    st = sptir_spmm(h, X, Y, feat, stream_);  // warm-up
    if (st == SPTIR_OK && hipEventRecord(e0, stream) != hipSuccess) st = note_hip_error(hipGetLastError(), "hipEventRecord");
    for (int32_t r = 0; r < reps && st == SPTIR_OK; ++r) st = sptir_spmm(h, X, Y, feat, stream_);
    if (st == SPTIR_OK && (hipEventRecord(e1, stream) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                           hipEventElapsedTime(&ms, e0, e1) != hipSuccess))
      st = note_hip_error(hipGetLastError(), "timing a candidate");
    if (st != SPTIR_OK) { sptir_hyb_destroy(h); goto done; }
    ms /= (float)reps;
    if (ms_per_candidate) ms_per_candidate[i] = ms;
    if (!best || ms < best_ms) {
      sptir_hyb_destroy(best);
      best = h; best_ms = ms; best_candidate = c_candidates[i];
    } else {
      sptir_hyb_destroy(h);
    }
  }
done:
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (st != SPTIR_OK) (void)hipStreamSynchronize(stream);
  if (X) free_(X, actx);
  if (Y) free_(Y, actx);
  if (st != SPTIR_OK) { sptir_hyb_destroy(best); return st; }
  *out = best;
  if (best_c) *best_c = best_candidate;
  return SPTIR_OK;
}
