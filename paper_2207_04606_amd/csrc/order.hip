// Launch order of the row blocks of every SpMM launch: longest chunk list first,
// so that the last wavefronts of a launch to finish are short ones (the row
// blocks of a power-law graph differ several-fold in work).  One stable radix
// sort over all launches at once: key = launch | (2^32 - 1 - list length),
// value = row block, so equal lengths stay in ascending row block order.
#include <cstring>

#include <rocprim/device/device_radix_sort.hpp>

#include "sptir_internal.h"

namespace sptir {
namespace {

__global__ void k_order_keys(int64_t n_groups, int32_t n_rb, const int64_t* __restrict__ rb_chunk_ptr,
                             unsigned long long* keys, int32_t* row_blocks) {
  const int64_t grp = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (grp >= n_groups) return;
  const int64_t len = rb_chunk_ptr[grp + 1] - rb_chunk_ptr[grp];
  const unsigned long long launch = (unsigned long long)(grp / n_rb);
  const unsigned long long clipped = len < 0xFFFFFFFFll ? (unsigned long long)len : 0xFFFFFFFFull;
  keys[grp] = (launch << 32) | (0xFFFFFFFFull - clipped);
  row_blocks[grp] = (int32_t)(grp % n_rb);
}

}  // namespace

sptir_status_t order_row_blocks(const int64_t* rb_chunk_ptr, int32_t n_launches, int32_t n_rb, int32_t* rb_order,
                                sptir_alloc_fn alloc, sptir_free_fn free_, void* actx, hipStream_t stream,
                                void** scratch_out) {
  *scratch_out = nullptr;
  const int64_t n = (int64_t)n_launches * n_rb;
  if (n <= 0) return SPTIR_OK;
  if (n > 0x7FFFFFFF) return SPTIR_ERR_OVERFLOW;
  unsigned int end_bit = 33;
  while (end_bit < 64 && (1ull << (end_bit - 32)) < (unsigned long long)n_launches) ++end_bit;
  size_t sort_bytes = 0;
  unsigned long long* no_keys = nullptr;
  int32_t* no_vals = nullptr;
  SPTIR_HIP(rocprim::radix_sort_pairs(nullptr, sort_bytes, no_keys, no_keys, no_vals, no_vals, (size_t)n, 0u, end_bit,
                                      stream));
  const size_t key_bytes = (sizeof(unsigned long long) * (size_t)n + 255) & ~(size_t)255;
  const size_t val_bytes = (sizeof(int32_t) * (size_t)n + 255) & ~(size_t)255;
  char* scratch = (char*)alloc(2 * key_bytes + val_bytes + (sort_bytes ? sort_bytes : 16), actx, stream);
  if (!scratch) return SPTIR_ERR_ALLOC;
  *scratch_out = scratch;  // the caller frees it once the stream has drained
  unsigned long long* keys_in = (unsigned long long*)scratch;
  unsigned long long* keys_out = (unsigned long long*)(scratch + key_bytes);
  int32_t* vals_in = (int32_t*)(scratch + 2 * key_bytes);
  void* sort_tmp = scratch + 2 * key_bytes + val_bytes;
  hipLaunchKernelGGL(k_order_keys, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, n, n_rb, rb_chunk_ptr,
                     keys_in, vals_in);
  SPTIR_HIP(hipGetLastError());
  SPTIR_HIP(rocprim::radix_sort_pairs(sort_tmp, sort_bytes, keys_in, keys_out, vals_in, rb_order, (size_t)n, 0u,
                                      end_bit, stream));
  return SPTIR_OK;
}

}  // namespace sptir
