// Launch order of the row blocks of every SpMM launch: longest chunk list first, so that the last wavefronts of a
// launch to finish are short ones (the row blocks of a power-law graph differ several-fold in work).  The launches
// are sorted independently of each other by a stable least-significant-digit radix sort, 8 bits a pass:
// key = 2^32 - 1 - list length, value = row block, so equal lengths stay in ascending row block order.  Only the
// digits that can differ are sorted: the caller says how long a list can be at most.
#include <cstring>

#include "sptir_internal.h"
#include "sptir_scan.h"

namespace sptir {
namespace {

constexpr int kSortTile = 1024;            // elements per workgroup and pass
constexpr int kSortRounds = kSortTile / 256;
constexpr int kDigits = 256;

__global__ void k_order_keys(int64_t n_groups, int32_t n_rb, const int64_t* __restrict__ rb_chunk_ptr,
                             uint32_t* __restrict__ keys, int32_t* __restrict__ row_blocks) {
  const int64_t grp = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (grp >= n_groups) return;
  const int64_t len = rb_chunk_ptr[grp + 1] - rb_chunk_ptr[grp];
  keys[grp] = 0xFFFFFFFFu - (len < 0xFFFFFFFFll ? (uint32_t)len : 0xFFFFFFFFu);
  row_blocks[grp] = (int32_t)(grp % n_rb);
}

// hist[(launch * 256 + digit) * tiles + tile] = elements of the tile with that digit; workgroup = launch * tiles + tile
__global__ __launch_bounds__(256) void k_sort_hist(const uint32_t* __restrict__ keys, int32_t n_rb, int tiles,
                                                   int shift, int32_t* __restrict__ hist) {
  __shared__ int count[kDigits];
  const int tile = blockIdx.x % tiles, launch = blockIdx.x / tiles;
  count[threadIdx.x] = 0;
  __syncthreads();
  const uint32_t* seg = keys + (int64_t)launch * n_rb;
#pragma unroll
  for (int r = 0; r < kSortRounds; ++r) {
    const int i = tile * kSortTile + r * 256 + threadIdx.x;
    if (i < n_rb) atomicAdd(&count[(seg[i] >> shift) & 255u], 1);
  }
  __syncthreads();
  hist[((int64_t)launch * kDigits + threadIdx.x) * tiles + tile] = count[threadIdx.x];
}

// `hist` scanned per launch (exclusive, digit-major): the first output position of each (digit, tile).  Elements
// keep their order inside a digit: the tile is walked 256 elements at a time, in order, and inside such a round a
// lane's rank is the number of lower lanes, then of lower wavefronts, with the same digit.
__global__ __launch_bounds__(256) void k_sort_scatter(const uint32_t* __restrict__ keys_in,
                                                      const int32_t* __restrict__ vals_in, int32_t n_rb, int tiles,
                                                      int shift, const int32_t* __restrict__ hist,
                                                      uint32_t* __restrict__ keys_out,
                                                      int32_t* __restrict__ vals_out) {
  __shared__ int base[kDigits];
  __shared__ int wave_cnt[4][kDigits];
  const int tile = blockIdx.x % tiles, launch = blockIdx.x / tiles;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  base[tid] = hist[((int64_t)launch * kDigits + tid) * tiles + tile];
#pragma unroll
  for (int w = 0; w < 4; ++w) wave_cnt[w][tid] = 0;
  __syncthreads();
  const int64_t seg0 = (int64_t)launch * n_rb;
  for (int r = 0; r < kSortRounds; ++r) {
    const int i = tile * kSortTile + r * 256 + tid;
    const bool valid = i < n_rb;
    const uint32_t key = valid ? keys_in[seg0 + i] : 0u;
    const int32_t val = valid ? vals_in[seg0 + i] : 0;
    const int digit = (int)((key >> shift) & 255u);
    unsigned long long peers = __ballot(valid);
#pragma unroll
    for (int bit = 0; bit < 8; ++bit) {
      const bool mine = (digit >> bit) & 1;
      const unsigned long long b = __ballot(mine);
      peers &= mine ? b : ~b;
    }
    const int rank_in_wave = __popcll(peers & ((1ull << lane) - 1ull));
    if (valid && rank_in_wave == 0) wave_cnt[wave][digit] = __popcll(peers);
    __syncthreads();
    if (valid) {
      int before = 0;
      for (int w = 0; w < wave; ++w) before += wave_cnt[w][digit];
      const int64_t at = seg0 + base[digit] + before + rank_in_wave;
      keys_out[at] = key;
      vals_out[at] = val;
    }
    __syncthreads();
    int all = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) { all += wave_cnt[w][tid]; wave_cnt[w][tid] = 0; }
    base[tid] += all;
    __syncthreads();
  }
}

}  // namespace

sptir_status_t order_row_blocks(const int64_t* rb_chunk_ptr, int32_t n_launches, int32_t n_rb, int64_t max_list_len,
                                int32_t* rb_order, sptir_alloc_fn alloc, sptir_free_fn free_, void* actx,
                                hipStream_t stream, void** scratch_out) {
  (void)free_;
  *scratch_out = nullptr;
  const int64_t n = (int64_t)n_launches * n_rb;
  if (n <= 0) return SPTIR_OK;
  if (n > 0x7FFFFFFF) return SPTIR_ERR_OVERFLOW;
  // the keys of a launch differ in the bits of (2^32 - 1 - length) below the highest bit a length can have
  int bits = 1;
  while (bits < 32 && ((int64_t)1 << bits) <= max_list_len) ++bits;
  const int passes = (bits + 7) / 8;
  const int64_t tiles = ((int64_t)n_rb + kSortTile - 1) / kSortTile;
  const int64_t n_hist = (int64_t)n_launches * kDigits * tiles;
  if (n_hist > 0x7FFFFFFF || tiles * n_launches > 0x7FFFFFFF) return SPTIR_ERR_OVERFLOW;
  const size_t key_bytes = (sizeof(uint32_t) * (size_t)n + 255) & ~(size_t)255;
  const size_t hist_bytes = (sizeof(int32_t) * (size_t)n_hist + 255) & ~(size_t)255;
  const size_t tot_bytes = (sizeof(int32_t) * (size_t)n_launches + 255) & ~(size_t)255;
  char* scratch = (char*)scratch_alloc(3 * key_bytes + hist_bytes + tot_bytes, alloc, actx, stream);
  if (!scratch) return SPTIR_ERR_ALLOC;
  *scratch_out = scratch;  // the caller gives it back (scratch_free) once the stream has drained
  uint32_t* keys[2] = {(uint32_t*)scratch, (uint32_t*)(scratch + key_bytes)};
  int32_t* other_vals = (int32_t*)(scratch + 2 * key_bytes);
  int32_t* hist = (int32_t*)(scratch + 3 * key_bytes);
  int32_t* totals = (int32_t*)(scratch + 3 * key_bytes + hist_bytes);
  // values ping-pong between rb_order and the scratch copy so that the last pass writes rb_order
  int32_t* vals[2];
  vals[passes % 2] = rb_order;
  vals[1 - passes % 2] = other_vals;
  hipLaunchKernelGGL(k_order_keys, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, n, n_rb, rb_chunk_ptr,
                     keys[0], vals[0]);
  for (int pass = 0; pass < passes; ++pass) {
    const int in = pass % 2, out = 1 - in;
    hipLaunchKernelGGL(k_sort_hist, dim3((unsigned)(tiles * n_launches)), dim3(256), 0, stream, keys[in], n_rb,
                       (int)tiles, 8 * pass, hist);
    hipLaunchKernelGGL(k_scan_sequences<int32_t>, dim3((unsigned)n_launches), dim3(kBuildBlock), 0, stream, hist,
                       (int32_t)(kDigits * tiles), totals);
    hipLaunchKernelGGL(k_sort_scatter, dim3((unsigned)(tiles * n_launches)), dim3(256), 0, stream, keys[in],
                       vals[in], n_rb, (int)tiles, 8 * pass, hist, keys[out], vals[out]);
  }
  SPTIR_HIP(hipGetLastError());
  return SPTIR_OK;
}

}  // namespace sptir
