// CSR -> hyb(c,k) format decomposition on the GPU (bucketing rule of section
// 4.2.1 of arXiv 2207.04606; the index inference that section 3.2.1 leaves to
// host pre-processing is done here by histogram -> scan -> stable scatter).
//
// Work unit: one thread per (row r, column partition p) pair, a workgroup per
// 256 consecutive rows of one partition.  A pair's row piece is the run of the
// row's (ascending) columns that fall in [p*w, (p+1)*w); its length l selects
// bin i = ceil(log2 l) (ELL bucket of width 2^i) or, for i > k, the remainder.
// Rows must appear in a bucket in ascending order, so placement is a stable
// multi-split: per-workgroup bin counts, an exclusive scan over workgroups per
// (partition, bin), and an in-workgroup rank from ballots.
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "sptir_internal.h"

namespace sptir {
namespace {

constexpr int kMaxBins = 32;  // k <= 30 -> bins 0..k plus the remainder bin k+1
constexpr int kWaves = kBuildBlock / 64;

struct BuildShape {
  int32_t n_rows, n_cols, c, k, w;
  int32_t nb;  // bins per partition = k + 2
  int32_t NB;  // row blocks = ceil(n_rows / 256)
  int32_t item_slots;
};

// first position q in [lo, hi) whose column is >= bound
__device__ __forceinline__ int lower_bound_col(const int32_t* __restrict__ indices, int lo, int hi, int64_t bound) {
  while (lo < hi) {
    int mid = lo + ((hi - lo) >> 1);
    if ((int64_t)indices[mid] < bound) lo = mid + 1; else hi = mid;
  }
  return lo;
}

// start and length of row r's piece in partition p
__device__ __forceinline__ void row_piece(const BuildShape& s, const int32_t* __restrict__ indptr,
                                          const int32_t* __restrict__ indices, int r, int p, int* lo, int* len) {
  int a = indptr[r], b = indptr[r + 1];
  int first = (p == 0) ? a : lower_bound_col(indices, a, b, (int64_t)p * s.w);
  int last = (p == s.c - 1) ? b : lower_bound_col(indices, first, b, (int64_t)(p + 1) * s.w);
  *lo = first;
  *len = last - first;
}

// bin of a piece of length l >= 1: smallest i with l <= 2^i, capped at k+1 (remainder)
__device__ __forceinline__ int bin_of_length(int l, int k) {
  int i = (l <= 1) ? 0 : 32 - __clz(l - 1);
  return i > k ? k + 1 : i;
}

// ---------------------------------------------------------------- validation
// flags[0]: indptr is not a non-decreasing prefix from 0 to nnz
// flags[1]: a column id outside [0, n_cols)
// flags[2]: number of positions q >= 1 with indices[q] <= indices[q-1]
// flags[3]: number of non-empty rows whose first column does not exceed the
//           column stored just before it (descents that are legal)
// Columns ascend strictly inside every row iff flags[2] == flags[3].
__global__ void k_validate_rows(int32_t n_rows, int64_t nnz, const int32_t* __restrict__ indptr,
                                const int32_t* __restrict__ indices, unsigned long long* flags) {
  int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= n_rows) return;
  int64_t a = indptr[r], b = indptr[r + 1];
  bool bad = (a < 0) || (b > nnz) || (a > b) || (r == 0 && a != 0) || (r == n_rows - 1 && b != nnz);
  if (bad) { flags[0] = 1; return; }
  if (a < b && a > 0 && indices[a] <= indices[a - 1]) atomicAdd(&flags[3], 1ull);
}

__global__ void k_validate_elems(int64_t nnz, int32_t n_cols, const int32_t* __restrict__ indices,
                                 unsigned long long* flags) {
  int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  bool descent = false, range = false;
  if (q < nnz) {
    int32_t col = indices[q];
    range = (col < 0) || (col >= n_cols);
    descent = (q > 0) && (col <= indices[q - 1]);
  }
  unsigned long long d = __ballot(descent);
  unsigned long long g = __ballot(range);
  if ((threadIdx.x & 63) == 0) {
    if (d) atomicAdd(&flags[2], (unsigned long long)__popcll(d));
    if (g) flags[1] = 1;
  }
}

// --------------------------------------------------------------------- count
// counts   [c][nb][NB] int32 : pieces of each bin per row block
// rem_nnz  [c][NB]     int64 : non-zeros sent to the remainder per row block
// rem_items[c][NB]     int64 : SpMM work items those pieces will need
__global__ __launch_bounds__(kBuildBlock) void k_count(BuildShape s, const int32_t* __restrict__ indptr,
                                                       const int32_t* __restrict__ indices, int32_t* counts,
                                                       int64_t* rem_nnz, int64_t* rem_items) {
  __shared__ int hist[kMaxBins];
  __shared__ unsigned long long sum_nnz, sum_items;
  int tid = threadIdx.x;
  int p = blockIdx.x / s.NB, rb = blockIdx.x % s.NB;
  if (tid < kMaxBins) hist[tid] = 0;
  if (tid == 0) { sum_nnz = 0; sum_items = 0; }
  __syncthreads();
  int r = rb * kBuildBlock + tid;
  if (r < s.n_rows) {
    int lo, l;
    row_piece(s, indptr, indices, r, p, &lo, &l);
    if (l > 0) {
      int bin = bin_of_length(l, s.k);
      atomicAdd(&hist[bin], 1);
      if (bin == s.k + 1) {
        atomicAdd(&sum_nnz, (unsigned long long)l);
        atomicAdd(&sum_items, (unsigned long long)((l + s.item_slots - 1) / s.item_slots));
      }
    }
  }
  __syncthreads();
  if (tid < s.nb) counts[((int64_t)p * s.nb + tid) * s.NB + rb] = hist[tid];
  if (tid == 0) {
    rem_nnz[(int64_t)p * s.NB + rb] = (int64_t)sum_nnz;
    rem_items[(int64_t)p * s.NB + rb] = (int64_t)sum_items;
  }
}

// ---------------------------------------------------------------------- scan
template <typename T>
__device__ __forceinline__ T wave_inclusive_scan(T v, int lane) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    T o = __shfl_up(v, d, 64);
    if (lane >= d) v += o;
  }
  return v;
}

// exclusive scan over the 256 threads of a workgroup; *total = sum of all
template <typename T>
__device__ __forceinline__ T block_exclusive_scan(T v, T* wave_sums /* [kWaves] shared */, T* total) {
  int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  T incl = wave_inclusive_scan(v, lane);
  __syncthreads();  // wave_sums may still be read from a previous call
  if (lane == 63) wave_sums[wave] = incl;
  __syncthreads();
  T base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    T ws = wave_sums[w];
    if (w < wave) base += ws;
    tot += ws;
  }
  *total = tot;
  return base + incl - v;
}

// One workgroup per sequence: data[seq*len .. +len) becomes its exclusive
// prefix, totals[seq] its sum.
template <typename T>
__global__ __launch_bounds__(kBuildBlock) void k_scan_sequences(T* data, int32_t len, T* totals) {
  __shared__ T wave_sums[kWaves];
  T* seq = data + (int64_t)blockIdx.x * len;
  T carry = 0;
  for (int32_t base = 0; base < len; base += kBuildBlock) {
    int32_t e = base + (int32_t)threadIdx.x;
    T v = (e < len) ? seq[e] : (T)0;
    T tot;
    T ex = block_exclusive_scan(v, wave_sums, &tot);
    if (e < len) seq[e] = carry + ex;
    carry += tot;
  }
  if (threadIdx.x == 0) totals[blockIdx.x] = carry;
}

// ------------------------------------------------------------------- scatter
struct ScatterArgs {
  const int32_t* indptr;
  const int32_t* indices;
  const float* values;
  const int32_t* counts;       // scanned: rank of the block's first piece of each bin
  const int64_t* rem_nnz;      // scanned
  const int64_t* rem_items;    // scanned
  const int64_t* bucket_row_ptr;
  const int64_t* bucket_slot_ptr;
  const int32_t* rem_part_ptr;
  const int64_t* rem_nnz_base;   // [c] first remainder nnz of each partition
  const int64_t* rem_item_base;  // [c] absolute index of the partition's first remainder work item
  int32_t* row_ids;
  int32_t* cols;
  float* vals;
  int64_t* rem_ptr;
  WorkItem* items;
  int64_t R, S, M, T;
};

// copies one row piece to `dst`: `len` real entries, then pads up to `width`
// (a pad repeats the last real column and holds +0.0f); lanes stride the piece
__device__ __forceinline__ void copy_piece(const ScatterArgs& a, int lo, int len, int width, int64_t dst, int first,
                                           int step) {
  for (int j = first; j < width; j += step) {
    int32_t col;
    float val;
    if (j < len) { col = a.indices[lo + j]; val = a.values[lo + j]; }
    else { col = a.indices[lo + len - 1]; val = 0.0f; }
    a.cols[dst + j] = col;
    a.vals[dst + j] = val;
  }
}

__global__ __launch_bounds__(kBuildBlock) void k_scatter(BuildShape s, ScatterArgs a) {
  __shared__ int wave_cnt[kWaves][kMaxBins];
  __shared__ long long wave_sums[kWaves];
  int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int p = blockIdx.x / s.NB, rb = blockIdx.x % s.NB;
  if (tid < kWaves * kMaxBins) (&wave_cnt[0][0])[tid] = 0;
  if (blockIdx.x == 0 && tid == 0) a.rem_ptr[a.M] = a.T;
  __syncthreads();

  int r = rb * kBuildBlock + tid;
  int lo = 0, l = 0, bin = -1;
  if (r < s.n_rows) {
    row_piece(s, a.indptr, a.indices, r, p, &lo, &l);
    if (l > 0) bin = bin_of_length(l, s.k);
  }
  // rank among the lanes of this wave that hold the same bin (stable: lower lanes first)
  int code = bin < 0 ? 63 : bin;
  unsigned long long peers = ~0ull;
#pragma unroll
  for (int bit = 0; bit < 6; ++bit) {
    bool mine = (code >> bit) & 1;
    unsigned long long b = __ballot(mine);
    peers &= mine ? b : ~b;
  }
  int rank_in_wave = __popcll(peers & ((1ull << lane) - 1ull));
  if (bin >= 0 && rank_in_wave == 0) wave_cnt[wave][bin] = __popcll(peers);

  // remainder pieces also need running sums of their lengths and work items
  bool is_rem = (bin == s.k + 1);
  long long my_nnz = is_rem ? l : 0;
  long long my_items = is_rem ? (l + s.item_slots - 1) / s.item_slots : 0;
  long long tot;
  long long nnz_before = block_exclusive_scan<long long>(my_nnz, wave_sums, &tot);
  long long items_before = block_exclusive_scan<long long>(my_items, wave_sums, &tot);
  // (block_exclusive_scan synchronises the workgroup, so wave_cnt is complete here)
  // Lanes without a piece stay alive with width 0: the wide copies below need all 64 lanes.
  int width = 0;
  int64_t dst = 0;
  if (bin >= 0) {
    int before = 0;
    for (int wv = 0; wv < wave; ++wv) before += wave_cnt[wv][bin];
    int64_t q = (int64_t)a.counts[((int64_t)p * s.nb + bin) * s.NB + rb] + before + rank_in_wave;
    if (!is_rem) {
      int64_t b = (int64_t)p * (s.k + 1) + bin;
      width = 1 << bin;
      a.row_ids[a.bucket_row_ptr[b] + q] = r;
      dst = a.bucket_slot_ptr[b] + q * width;
    } else {
      int64_t m = (int64_t)a.rem_part_ptr[p] + q;
      int64_t t0 = a.rem_nnz_base[p] + a.rem_nnz[(int64_t)p * s.NB + rb] + nnz_before;
      a.row_ids[a.R + m] = r;
      a.rem_ptr[m] = t0;
      width = l;
      dst = a.S + t0;
      // the piece's SpMM work items: item_slots non-zeros each, one row
      int64_t it = a.rem_item_base[p] + a.rem_items[(int64_t)p * s.NB + rb] + items_before;
      for (int off = 0; off < l; off += s.item_slots, ++it) {
        int cnt = min(s.item_slots, l - off);
        WorkItem w;
        w.slot0 = dst + off;
        w.row0 = (int32_t)(a.R + m);
        w.meta = (uint32_t)kRemLog2W | ((uint32_t)cnt << 6);
        a.items[it] = w;
      }
    }
  }
  // short pieces are copied by their own lane, long ones by the whole wave
  constexpr int kOwnLaneMax = 4;
  if (width > 0 && width <= kOwnLaneMax) copy_piece(a, lo, l, width, dst, 0, 1);
  unsigned long long wide = __ballot(width > kOwnLaneMax);
  while (wide) {
    int src = __ffsll((long long)wide) - 1;
    wide &= wide - 1;
    int lo_s = __shfl(lo, src, 64), l_s = __shfl(l, src, 64), width_s = __shfl(width, src, 64);
    long long dst_s = __shfl((long long)dst, src, 64);
    copy_piece(a, lo_s, l_s, width_s, dst_s, lane, 64);
  }
}

// ELL work items: bucket b contributes ceil(slots_b / item_slots) items, stored
// from items[item_base[b]]; item_prefix is the dense prefix used to map a
// thread to its bucket.
__global__ void k_make_ell_items(int32_t B, int32_t k, int32_t item_slots, const int64_t* __restrict__ item_prefix,
                                 const int64_t* __restrict__ item_base, const int64_t* __restrict__ bucket_row_ptr,
                                 const int64_t* __restrict__ bucket_slot_ptr, WorkItem* items) {
  int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (u >= item_prefix[B]) return;
  int lo = 0, hi = B;  // last b with item_prefix[b] <= u
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (item_prefix[mid] <= u) lo = mid; else hi = mid;
  }
  int b = lo, i = b % (k + 1);
  int64_t j = u - item_prefix[b];
  int64_t off = j * item_slots;
  int64_t slots = bucket_slot_ptr[b + 1] - bucket_slot_ptr[b];
  int64_t cnt = slots - off < item_slots ? slots - off : item_slots;
  WorkItem w;
  w.slot0 = bucket_slot_ptr[b] + off;
  w.row0 = (int32_t)(bucket_row_ptr[b] + (off >> i));
  w.meta = (uint32_t)i | ((uint32_t)cnt << 6);
  items[item_base[b] + j] = w;
}

// --------------------------------------------------------------- host helpers
struct Blob {  // bump allocator over one device allocation
  char* base = nullptr;
  size_t size = 0;
  size_t reserve(size_t bytes) {
    size_t off = size;
    size = (size + bytes + 255) & ~(size_t)255;
    return off;
  }
};

int item_slots_setting() {
  const char* e = getenv("SPTIR_ITEM_SLOTS");
  long v = e ? atol(e) : 1024;
  if (v < 64 || v > 65536 || (v & (v - 1))) v = 1024;
  return (int)v;
}

}  // namespace
}  // namespace sptir

using namespace sptir;

extern "C" sptir_status_t sptir_hyb_build(const sptir_csr_t* csr, int32_t n_col_parts, int32_t max_bucket_log2,
                                          void* stream_, sptir_hyb_t** out) {
  if (!csr || !out) return SPTIR_ERR_INVALID_ARG;
  if (csr->n_rows < 0 || csr->n_cols < 0 || csr->nnz < 0) return SPTIR_ERR_INVALID_ARG;
  if (n_col_parts < 1 || max_bucket_log2 < 0 || max_bucket_log2 > 30) return SPTIR_ERR_INVALID_ARG;
  if (csr->nnz >= ((int64_t)1 << 31)) return SPTIR_ERR_OVERFLOW;
  if (!csr->indptr || (csr->nnz > 0 && (!csr->indices || !csr->values))) return SPTIR_ERR_INVALID_ARG;
  if (csr->nnz > 0 && (csr->n_rows == 0 || csr->n_cols == 0)) return SPTIR_ERR_INVALID_ARG;
  hipStream_t stream = (hipStream_t)stream_;

  BuildShape s;
  s.n_rows = csr->n_rows; s.n_cols = csr->n_cols; s.c = n_col_parts; s.k = max_bucket_log2;
  s.w = (int32_t)(((int64_t)csr->n_cols + n_col_parts - 1) / n_col_parts);
  s.nb = s.k + 2;
  s.NB = (s.n_rows + kBuildBlock - 1) / kBuildBlock;
  s.item_slots = item_slots_setting();
  const int64_t n_pair_blocks = (int64_t)s.NB * s.c;
  if (n_pair_blocks > 0x7FFFFFFF) return SPTIR_ERR_OVERFLOW;
  const int64_t B = (int64_t)s.c * (s.k + 1);
  if (B > 0x7FFFFFFF) return SPTIR_ERR_OVERFLOW;

  sptir_alloc_fn alloc; sptir_free_fn free_; void* actx;
  current_allocator(&alloc, &free_, &actx);

  // ---- temporary device storage (one blob)
  Blob tmp;
  const size_t o_flags = tmp.reserve(4 * sizeof(unsigned long long));
  const size_t o_counts = tmp.reserve(sizeof(int32_t) * (size_t)s.c * s.nb * (size_t)(s.NB ? s.NB : 1));
  const size_t o_rnnz = tmp.reserve(sizeof(int64_t) * (size_t)s.c * (size_t)(s.NB ? s.NB : 1));
  const size_t o_ritems = tmp.reserve(sizeof(int64_t) * (size_t)s.c * (size_t)(s.NB ? s.NB : 1));
  const size_t o_tot_bins = tmp.reserve(sizeof(int32_t) * (size_t)s.c * s.nb);
  const size_t o_tot_rnnz = tmp.reserve(sizeof(int64_t) * (size_t)s.c);
  const size_t o_tot_ritems = tmp.reserve(sizeof(int64_t) * (size_t)s.c);
  const size_t o_rnnz_base = tmp.reserve(sizeof(int64_t) * (size_t)s.c);
  const size_t o_ritem_base = tmp.reserve(sizeof(int64_t) * (size_t)s.c);
  const size_t o_item_prefix = tmp.reserve(sizeof(int64_t) * (size_t)(B + 1));
  const size_t o_item_base = tmp.reserve(sizeof(int64_t) * (size_t)(B + 1));
  tmp.base = (char*)alloc(tmp.size, actx, stream);
  if (!tmp.base) return SPTIR_ERR_ALLOC;

  sptir_hyb* h = new (std::nothrow) sptir_hyb();
  if (!h) { free_(tmp.base, actx); return SPTIR_ERR_ALLOC; }
  memset(h, 0, sizeof(*h));
  h->alloc = alloc; h->free_ = free_; h->alloc_ctx = actx;
  h->n_rows = s.n_rows; h->n_cols = s.n_cols; h->c = s.c; h->k = s.k; h->w = s.w;
  h->nnz = csr->nnz; h->B = B; h->item_slots = s.item_slots;

  // every exit after this point goes through `fail`
  sptir_status_t st = SPTIR_OK;
#define BUILD_HIP(call)                                              \
  do {                                                               \
    hipError_t e_ = (call);                                          \
    if (e_ != hipSuccess) { st = note_hip_error(e_, #call); goto fail; } \
  } while (0)

  {
    unsigned long long* d_flags = (unsigned long long*)(tmp.base + o_flags);
    int32_t* d_counts = (int32_t*)(tmp.base + o_counts);
    int64_t* d_rnnz = (int64_t*)(tmp.base + o_rnnz);
    int64_t* d_ritems = (int64_t*)(tmp.base + o_ritems);
    int32_t* d_tot_bins = (int32_t*)(tmp.base + o_tot_bins);
    int64_t* d_tot_rnnz = (int64_t*)(tmp.base + o_tot_rnnz);
    int64_t* d_tot_ritems = (int64_t*)(tmp.base + o_tot_ritems);
    int64_t* d_rnnz_base = (int64_t*)(tmp.base + o_rnnz_base);
    int64_t* d_ritem_base = (int64_t*)(tmp.base + o_ritem_base);
    int64_t* d_item_prefix = (int64_t*)(tmp.base + o_item_prefix);
    int64_t* d_item_base = (int64_t*)(tmp.base + o_item_base);

    // ---- validation of the CSR input
    unsigned long long flags[4] = {0, 0, 0, 0};
    BUILD_HIP(hipMemsetAsync(d_flags, 0, sizeof(flags), stream));
    if (s.n_rows > 0)
      hipLaunchKernelGGL(k_validate_rows, dim3((s.n_rows + 255) / 256), dim3(256), 0, stream, s.n_rows, csr->nnz,
                         csr->indptr, csr->indices, d_flags);
    if (csr->nnz > 0)
      hipLaunchKernelGGL(k_validate_elems, dim3((unsigned)((csr->nnz + 255) / 256)), dim3(256), 0, stream, csr->nnz,
                         s.n_cols, csr->indices, d_flags);
    BUILD_HIP(hipGetLastError());
    BUILD_HIP(hipMemcpyAsync(flags, d_flags, sizeof(flags), hipMemcpyDeviceToHost, stream));
    BUILD_HIP(hipStreamSynchronize(stream));
    if (s.n_rows == 0) {
      int32_t first = 0;
      BUILD_HIP(hipMemcpyAsync(&first, csr->indptr, sizeof(int32_t), hipMemcpyDeviceToHost, stream));
      BUILD_HIP(hipStreamSynchronize(stream));
      if (first != 0) flags[0] = 1;
    }
    if (flags[0]) { st = SPTIR_ERR_INVALID_ARG; goto fail; }
    if (flags[1] || flags[2] != flags[3]) { st = SPTIR_ERR_UNSORTED; goto fail; }

    // ---- histogram and scans
    std::vector<int32_t> tot_bins((size_t)s.c * s.nb, 0);
    std::vector<int64_t> tot_rnnz((size_t)s.c, 0), tot_ritems((size_t)s.c, 0);
    if (s.NB > 0) {
      hipLaunchKernelGGL(k_count, dim3((unsigned)n_pair_blocks), dim3(kBuildBlock), 0, stream, s, csr->indptr,
                         csr->indices, d_counts, d_rnnz, d_ritems);
      hipLaunchKernelGGL(k_scan_sequences<int32_t>, dim3((unsigned)(s.c * s.nb)), dim3(kBuildBlock), 0, stream,
                         d_counts, s.NB, d_tot_bins);
      hipLaunchKernelGGL(k_scan_sequences<long long>, dim3((unsigned)s.c), dim3(kBuildBlock), 0, stream,
                         (long long*)d_rnnz, s.NB, (long long*)d_tot_rnnz);
      hipLaunchKernelGGL(k_scan_sequences<long long>, dim3((unsigned)s.c), dim3(kBuildBlock), 0, stream,
                         (long long*)d_ritems, s.NB, (long long*)d_tot_ritems);
      BUILD_HIP(hipGetLastError());
      BUILD_HIP(hipMemcpyAsync(tot_bins.data(), d_tot_bins, sizeof(int32_t) * tot_bins.size(),
                               hipMemcpyDeviceToHost, stream));
      BUILD_HIP(hipMemcpyAsync(tot_rnnz.data(), d_tot_rnnz, sizeof(int64_t) * s.c, hipMemcpyDeviceToHost, stream));
      BUILD_HIP(hipMemcpyAsync(tot_ritems.data(), d_tot_ritems, sizeof(int64_t) * s.c, hipMemcpyDeviceToHost,
                               stream));
      BUILD_HIP(hipStreamSynchronize(stream));
    }

    // ---- sizes and the small prefix arrays (host)
    std::vector<int64_t> row_ptr((size_t)B + 1, 0), slot_ptr((size_t)B + 1, 0);
    std::vector<int64_t> item_prefix((size_t)B + 1, 0), item_base((size_t)B + 1, 0);
    std::vector<int32_t> rem_part_ptr((size_t)s.c + 1, 0);
    std::vector<int64_t> rnnz_base((size_t)s.c, 0), ritem_base((size_t)s.c, 0);
    int64_t M = 0, T = 0, n_items = 0;
    for (int32_t p = 0; p < s.c; ++p) {
      for (int32_t i = 0; i <= s.k; ++i) {
        int64_t b = (int64_t)p * (s.k + 1) + i;
        int64_t rows = tot_bins[(size_t)p * s.nb + i];
        int64_t slots = rows << i;
        row_ptr[b + 1] = row_ptr[b] + rows;
        slot_ptr[b + 1] = slot_ptr[b] + slots;
        int64_t its = (slots + s.item_slots - 1) / s.item_slots;
        item_prefix[b + 1] = item_prefix[b] + its;
        item_base[b] = n_items;
        n_items += its;
      }
      rnnz_base[p] = T;
      ritem_base[p] = n_items;
      M += tot_bins[(size_t)p * s.nb + s.k + 1];
      T += tot_rnnz[p];
      n_items += tot_ritems[p];
      if (M > 0x7FFFFFFF) { st = SPTIR_ERR_OVERFLOW; goto fail; }
      rem_part_ptr[p + 1] = (int32_t)M;
    }
    h->R = row_ptr[B]; h->S = slot_ptr[B]; h->M = M; h->T = T; h->n_items = n_items;
    if (h->R + h->M > 0x7FFFFFFF) { st = SPTIR_ERR_OVERFLOW; goto fail; }

    // ---- the handle's device arrays
    struct { void** p; size_t bytes; } wanted[] = {
        {(void**)&h->bucket_row_ptr, sizeof(int64_t) * (size_t)(B + 1)},
        {(void**)&h->bucket_slot_ptr, sizeof(int64_t) * (size_t)(B + 1)},
        {(void**)&h->rem_part_ptr, sizeof(int32_t) * (size_t)(s.c + 1)},
        {(void**)&h->rem_ptr, sizeof(int64_t) * (size_t)(M + 1)},
        {(void**)&h->row_ids, sizeof(int32_t) * (size_t)(h->R + M)},
        {(void**)&h->cols, sizeof(int32_t) * (size_t)(h->S + T)},
        {(void**)&h->vals, sizeof(float) * (size_t)(h->S + T)},
        {(void**)&h->items, sizeof(WorkItem) * (size_t)n_items},
    };
    for (auto& wnt : wanted) {
      size_t bytes = wnt.bytes ? wnt.bytes : 16;
      *wnt.p = alloc(bytes, actx, stream);
      if (!*wnt.p) { st = SPTIR_ERR_ALLOC; goto fail; }
      h->device_bytes += bytes;
    }
    BUILD_HIP(hipMemcpyAsync(h->bucket_row_ptr, row_ptr.data(), sizeof(int64_t) * (B + 1), hipMemcpyHostToDevice,
                             stream));
    BUILD_HIP(hipMemcpyAsync(h->bucket_slot_ptr, slot_ptr.data(), sizeof(int64_t) * (B + 1), hipMemcpyHostToDevice,
                             stream));
    BUILD_HIP(hipMemcpyAsync(h->rem_part_ptr, rem_part_ptr.data(), sizeof(int32_t) * (s.c + 1),
                             hipMemcpyHostToDevice, stream));
    BUILD_HIP(hipMemcpyAsync(d_rnnz_base, rnnz_base.data(), sizeof(int64_t) * s.c, hipMemcpyHostToDevice, stream));
    BUILD_HIP(hipMemcpyAsync(d_ritem_base, ritem_base.data(), sizeof(int64_t) * s.c, hipMemcpyHostToDevice, stream));
    BUILD_HIP(hipMemcpyAsync(d_item_prefix, item_prefix.data(), sizeof(int64_t) * (B + 1), hipMemcpyHostToDevice,
                             stream));
    BUILD_HIP(hipMemcpyAsync(d_item_base, item_base.data(), sizeof(int64_t) * (B + 1), hipMemcpyHostToDevice,
                             stream));

    // ---- stable scatter and work-item list
    if (s.NB > 0) {
      ScatterArgs a;
      a.indptr = csr->indptr; a.indices = csr->indices; a.values = csr->values;
      a.counts = d_counts; a.rem_nnz = d_rnnz; a.rem_items = d_ritems;
      a.bucket_row_ptr = h->bucket_row_ptr; a.bucket_slot_ptr = h->bucket_slot_ptr;
      a.rem_part_ptr = h->rem_part_ptr; a.rem_nnz_base = d_rnnz_base; a.rem_item_base = d_ritem_base;
      a.row_ids = h->row_ids; a.cols = h->cols; a.vals = h->vals; a.rem_ptr = h->rem_ptr; a.items = h->items;
      a.R = h->R; a.S = h->S; a.M = M; a.T = T;
      hipLaunchKernelGGL(k_scatter, dim3((unsigned)n_pair_blocks), dim3(kBuildBlock), 0, stream, s, a);
    } else {
      int64_t zero = 0;
      BUILD_HIP(hipMemcpyAsync(h->rem_ptr, &zero, sizeof(int64_t), hipMemcpyHostToDevice, stream));
    }
    if (item_prefix[B] > 0) {
      int64_t blocks = (item_prefix[B] + 255) / 256;
      if (blocks > 0x7FFFFFFF) { st = SPTIR_ERR_OVERFLOW; goto fail; }
      hipLaunchKernelGGL(k_make_ell_items, dim3((unsigned)blocks), dim3(256), 0, stream, (int32_t)B, s.k,
                         s.item_slots, d_item_prefix, d_item_base, h->bucket_row_ptr, h->bucket_slot_ptr, h->items);
    }
    BUILD_HIP(hipGetLastError());
    BUILD_HIP(hipStreamSynchronize(stream));
  }
  free_(tmp.base, actx);
  *out = h;
  return SPTIR_OK;

fail:
  (void)hipStreamSynchronize(stream);
  free_(tmp.base, actx);
  sptir_hyb_destroy(h);
  return st;
#undef BUILD_HIP
}
