// Internal declarations shared by the translation units of libsptir.so.
#ifndef SPTIR_INTERNAL_H_
#define SPTIR_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sptir.h"

namespace sptir {

// One wavefront's share of an SpMM launch: `count` consecutive stored slots of
// the fused (cols, vals) arrays starting at `slot0`.  Slot o of the item
// belongs to row_ids[row0 + (o >> log2w)]; for an ELL bucket log2w is the
// bucket's i (section 4.2.1: width 2^i), for a piece of the CSR remainder it
// is 31 so that the whole item is one row.
struct WorkItem {
  int64_t slot0;
  int32_t row0;
  uint32_t meta;  // bits 0..5 log2w, bits 6..31 count
};
static_assert(sizeof(WorkItem) == 16, "WorkItem must stay 16 bytes");

constexpr int kRemLog2W = 31;
constexpr int kBuildBlock = 256;  // rows per workgroup in the builder kernels

}  // namespace sptir

// The handle behind sptir_hyb_t.  ELL and remainder share three device
// allocations so that one SpMM launch can walk both:
//   row_ids = [ELL_ROW | REM_ROW], cols = [ELL_COL | REM_COL], vals likewise.
struct sptir_hyb {
  int32_t n_rows, n_cols, c, k, w;
  int64_t nnz;
  int64_t B, R, S, M, T;
  int64_t* bucket_row_ptr;   // device [B+1]
  int64_t* bucket_slot_ptr;  // device [B+1]
  int32_t* rem_part_ptr;     // device [c+1]
  int64_t* rem_ptr;          // device [M+1]
  int32_t* row_ids;          // device [R+M]
  int32_t* cols;             // device [S+T]
  float* vals;               // device [S+T]
  sptir::WorkItem* items;    // device [n_items]
  int64_t n_items;
  int32_t item_slots;
  size_t device_bytes;
  sptir_alloc_fn alloc;
  sptir_free_fn free_;
  void* alloc_ctx;
};

namespace sptir {

// allocator currently installed (api.hip)
void current_allocator(sptir_alloc_fn* a, sptir_free_fn* f, void** ctx);
void* default_alloc(size_t bytes, void* ctx, void* stream);
void default_free(void* p, void* ctx);

// records a failed HIP call for sptir_last_hip_error(); returns SPTIR_ERR_HIP
sptir_status_t note_hip_error(hipError_t e, const char* what);

#define SPTIR_HIP(call)                                                   \
  do {                                                                    \
    hipError_t e_ = (call);                                               \
    if (e_ != hipSuccess) return ::sptir::note_hip_error(e_, #call);      \
  } while (0)

}  // namespace sptir

#endif  // SPTIR_INTERNAL_H_
