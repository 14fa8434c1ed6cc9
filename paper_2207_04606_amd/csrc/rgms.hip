// Relational gather-matmul-scatter (RGMS, section 4.4 of arXiv 2207.04606):
//     Y[i,l] = sum_r sum_j sum_k A[r,i,j] * X[j,k] * W[r,k,l].
// The paper decomposes every relation's matrix into hyb(1, 5) (a "3-D hyb"),
// pins W[r] on chip for each ELL sub-matrix of relation r, gathers the rows
// of X it needs, multiplies on the matrix cores and scatters into Y, all in
// one kernel, so that T[r] = X W[r] never exists in memory.
//
// Here A arrives as one CSR over stacked rows r*n + i, and its 3-D hyb is the
// ordinary hyb(1, k) of that stacked matrix: bucket i holds the stacked rows
// with 2^(i-1) < l <= 2^i entries, ascending, hence relation after relation.
// The buckets are cut into tiles of 32 stacked rows of one relation (pieces
// longer than 2^k go to the remainder and are cut into 32-entry segments).
// One wavefront takes a tile:
//   gather     eight 8-lane groups sum a[i,j] * X[j,:] for four rows each
//              (aggregating before the product is the same sum and leaves one
//              matrix row per stacked row instead of one per non-zero);
//              the 32 x d_in block Z goes to LDS;
//   matmul     Z (32 x d_in) times W[r] (d_in x d_out) with
//              v_mfma_f32_32x32x2_f32, float32 throughout, W[r] read from L2;
//   scatter    float atomic adds of the 32 x 32 results into the rows of Y
//              (a row of Y collects from every relation and bucket, in no
//              fixed order: results agree to rounding, not bit for bit).
//              These atomics execute beyond L2 and bound the kernel at about
//              1 TB/s of added bytes; ordering the tiles by destination row
//              was measured to change nothing.
// Y is zero-filled first by a kernel of its own (the operator overwrites Y).
#include <string.h>

#include <algorithm>
#include <new>
#include <vector>

#include "sptir_internal.h"
#include "sptir_scan.h"

namespace sptir {
namespace {

struct RgmsTile {
  int64_t slot0;      // first slot of the tile's first row in the fused (cols, vals) arrays
  int32_t row0;       // index of the tile's first row in row_ids
  int32_t n_rows;     // 1..32 rows (ELL) or 32-entry segments (remainder)
  int32_t log2w;      // ELL: log2 of the bucket width; -1: segments of one remainder piece
  int32_t rel;
  int32_t last_len;   // remainder: entries in the tile's last segment (1..32)
  int32_t pad_;
};
static_assert(sizeof(RgmsTile) == 32, "RgmsTile must stay 32 bytes");

constexpr int kRgmsWaves = 4;
typedef float floatx16 __attribute__((ext_vector_type(16)));

struct RgmsArgs {
  const RgmsTile* tiles;
  const int32_t* row_ids;
  const int32_t* cols;
  const float* vals;
  const float* X;
  const float* W;
  float* Y;
  int64_t n_tiles;
  int32_t n_rows;  // rows of Y = rows per relation
  int32_t d_in, d_out;
};

__global__ void k_fill_zero(float* p, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = 0.f;
}

// bounds[(i * (n_rel + 1)) + r] = first position in [lo_i, hi_i) of row_ids whose stacked row is >= r * n_rows,
// for every list i (the k+1 ELL buckets, then the remainder)
__global__ void k_relation_bounds(int32_t n_lists, int32_t n_rel, int32_t n_rows, const int64_t* __restrict__ list_lo,
                                  const int64_t* __restrict__ list_hi, const int32_t* __restrict__ row_ids,
                                  int64_t* bounds) {
  int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n_lists * (n_rel + 1)) return;
  int i = t / (n_rel + 1), r = t % (n_rel + 1);
  int64_t lo = list_lo[i], hi = list_hi[i];
  const int64_t bound = (int64_t)r * n_rows;
  while (lo < hi) {
    int64_t mid = lo + ((hi - lo) >> 1);
    if ((int64_t)row_ids[mid] < bound) lo = mid + 1; else hi = mid;
  }
  bounds[t] = lo;
}

// TIN float4 per lane cover d_in = 32 * TIN floats of a row of X
template <int TIN>
__global__ __launch_bounds__(64 * kRgmsWaves) void k_rgms(RgmsArgs a) {
  constexpr int kDin = 32 * TIN;
  constexpr int kZStride = kDin + 1;  // odd stride: the column reads of the matrix product hit 32 different banks
  __shared__ float z_all[kRgmsWaves][32 * kZStride];
  const int lane = threadIdx.x & 63, g = lane >> 3, fl = lane & 7;
  const int wave = threadIdx.x >> 6;
  const int64_t t = (int64_t)blockIdx.x * kRgmsWaves + wave;
  if (t >= a.n_tiles) return;  // (no barriers below: the wavefronts of a workgroup are independent)
  const RgmsTile tile = a.tiles[t];
  float* z = z_all[wave];
  const bool ell = tile.log2w >= 0;
  const int width = ell ? (1 << tile.log2w) : 32;

  // ---- gather: row m*8 + g of the tile for m = 0..3
#pragma unroll 1
  for (int m = 0; m < 4; ++m) {
    const int row = m * 8 + g;
    float4 acc[TIN];
#pragma unroll
    for (int q = 0; q < TIN; ++q) acc[q] = make_float4(0.f, 0.f, 0.f, 0.f);
    // (the trip counts below are the same for every lane group of the wavefront)
    const bool row_in = row < tile.n_rows;
    const int len = !row_in ? 0 : (ell || row < tile.n_rows - 1) ? width : tile.last_len;
    const int64_t base = tile.slot0 + (int64_t)(row_in ? row : 0) * width;
    for (int s0 = 0; s0 < width; s0 += 8) {
      const int j = s0 + fl;
      const bool in = j < len;
      const int col_reg = a.cols[base + (in ? j : 0)];
      const float val_reg = in ? a.vals[base + j] : 0.f;
      const int steps = min(8, width - s0);
      for (int u = 0; u < steps; ++u) {
        const int c = __shfl(col_reg, g * 8 + u, 64);
        const float v = __shfl(val_reg, g * 8 + u, 64);
        const float* xr = a.X + (size_t)c * kDin + 4 * fl;
#pragma unroll
        for (int q = 0; q < TIN; ++q) {
          const float4 x = *reinterpret_cast<const float4*>(xr + 32 * q);
          acc[q].x = fmaf(v, x.x, acc[q].x); acc[q].y = fmaf(v, x.y, acc[q].y);
          acc[q].z = fmaf(v, x.z, acc[q].z); acc[q].w = fmaf(v, x.w, acc[q].w);
        }
      }
    }
#pragma unroll
    for (int q = 0; q < TIN; ++q) {
      float* zr = z + row * kZStride + 32 * q + 4 * fl;
      zr[0] = acc[q].x; zr[1] = acc[q].y; zr[2] = acc[q].z; zr[3] = acc[q].w;
    }
  }
  // the stacked row of every tile row -> its row of Y (lanes 0..31 hold rows 0..31)
  int y_row_reg = 0;
  if (lane < tile.n_rows) {
    const int stacked = a.row_ids[tile.row0 + (ell ? lane : 0)];
    y_row_reg = stacked - tile.rel * a.n_rows;
  }

  // ---- matmul and scatter, 32 columns of Y at a time
  const float* w_rel = a.W + (size_t)tile.rel * kDin * (size_t)a.d_out;
  const int mi = lane & 31, kh = lane >> 5;  // this lane's row of A / column of B, and which of the two k it holds
  for (int n0 = 0; n0 < a.d_out; n0 += 32) {
    floatx16 d;
#pragma unroll
    for (int v = 0; v < 16; ++v) d[v] = 0.f;
#pragma unroll 4
    for (int kk = 0; kk < kDin / 2; ++kk) {
      const float av = z[mi * kZStride + 2 * kk + kh];                      // A[mi][2kk + kh]
      const float bv = w_rel[(size_t)(2 * kk + kh) * a.d_out + n0 + mi];    // B[2kk + kh][mi]
      d = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, d, 0, 0, 0);
    }
    // d[v] = D[8*(v/4) + 4*kh + v%4][mi]
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = 8 * (v >> 2) + 4 * kh + (v & 3);
      const int y_row = __shfl(y_row_reg, row, 64);
      if (row < tile.n_rows) atomicAdd(a.Y + (size_t)y_row * a.d_out + n0 + mi, d[v]);
    }
  }
}

}  // namespace
}  // namespace sptir

// The handle behind sptir_rgms_t.
struct sptir_rgms_handle {
  int32_t n_rel, n_rows, n_cols, k;
  int64_t nnz;
  sptir_hyb_t* hyb;  // hyb(1, k) of the stacked matrix (canonical arrays only)
  sptir::RgmsTile* tiles;
  int64_t n_tiles;
  size_t device_bytes;
  sptir_alloc_fn alloc;
  sptir_free_fn free_;
  void* alloc_ctx;
};

using namespace sptir;

extern "C" sptir_status_t sptir_rgms_destroy(sptir_rgms_t* p) {
  if (!p) return SPTIR_OK;
  if (p->tiles) p->free_(p->tiles, p->alloc_ctx);
  sptir_hyb_destroy(p->hyb);
  delete p;
  return SPTIR_OK;
}

extern "C" sptir_status_t sptir_rgms_info(const sptir_rgms_t* p, sptir_rgms_info_t* out) {
  if (!p || !out) return SPTIR_ERR_INVALID_ARG;
  sptir_hyb_info_t hi;
  sptir_status_t st = sptir_hyb_info(p->hyb, &hi);
  if (st != SPTIR_OK) return st;
  sptir_rgms_info_t o;
  o.n_relations = p->n_rel; o.n_rows = p->n_rows; o.n_cols = p->n_cols; o.max_bucket_log2 = p->k;
  o.nnz = p->nnz; o.n_stacked_rows_stored = hi.n_ell_rows + hi.n_rem_pieces; o.n_pad_slots = hi.n_pad_slots;
  o.n_tiles = p->n_tiles; o.device_bytes = (int64_t)p->device_bytes + hi.device_bytes;
  *out = o;
  return SPTIR_OK;
}

extern "C" sptir_status_t sptir_rgms_build(const sptir_csr_t* stacked, int32_t n_relations, int32_t max_bucket_log2,
                                           void* stream_, sptir_rgms_t** out) {
  if (!stacked || !out || n_relations < 1) return SPTIR_ERR_INVALID_ARG;
  if (stacked->n_rows < 0 || stacked->n_rows % n_relations != 0) return SPTIR_ERR_INVALID_ARG;
  const int32_t k = max_bucket_log2 < 0 ? 5 : max_bucket_log2;  // the paper decomposes every relation as hyb(1, 5)
  if (k > 5) return SPTIR_ERR_INVALID_ARG;  // a tile row holds at most 32 entries
  hipStream_t stream = (hipStream_t)stream_;
  sptir_rgms_handle* p = new (std::nothrow) sptir_rgms_handle();
  if (!p) return SPTIR_ERR_ALLOC;
  memset(p, 0, sizeof(*p));
  current_allocator(&p->alloc, &p->free_, &p->alloc_ctx);
  p->n_rel = n_relations; p->n_rows = stacked->n_rows / n_relations; p->n_cols = stacked->n_cols; p->k = k;
  p->nnz = stacked->nnz;
  sptir_status_t st = hyb_build_impl(stacked, 1, k, stream_, &p->hyb, false);
  if (st != SPTIR_OK) { delete p; return st; }

  const sptir_hyb* h = p->hyb;
  const int n_lists = k + 2;  // the ELL buckets and the remainder
  std::vector<int64_t> bucket_row_ptr((size_t)k + 2), bucket_slot_ptr((size_t)k + 2), rem_ptr((size_t)h->M + 1);
  std::vector<int64_t> list_lo((size_t)n_lists), list_hi((size_t)n_lists), bounds((size_t)n_lists * (n_relations + 1));
  std::vector<RgmsTile> tiles;
  int64_t* d_lists = nullptr;
  int64_t* d_bounds = nullptr;
#define RGMS_HIP(call)                                                 \
  do {                                                                 \
    hipError_t e_ = (call);                                            \
    if (e_ != hipSuccess) { st = note_hip_error(e_, #call); goto fail; } \
  } while (0)
  RGMS_HIP(hipMemcpyAsync(bucket_row_ptr.data(), h->bucket_row_ptr, sizeof(int64_t) * (k + 2), hipMemcpyDeviceToHost,
                          stream));
  RGMS_HIP(hipMemcpyAsync(bucket_slot_ptr.data(), h->bucket_slot_ptr, sizeof(int64_t) * (k + 2), hipMemcpyDeviceToHost,
                          stream));
  RGMS_HIP(hipMemcpyAsync(rem_ptr.data(), h->rem_ptr, sizeof(int64_t) * (h->M + 1), hipMemcpyDeviceToHost, stream));
  RGMS_HIP(hipStreamSynchronize(stream));
  for (int i = 0; i <= k; ++i) { list_lo[i] = bucket_row_ptr[i]; list_hi[i] = bucket_row_ptr[i + 1]; }
  list_lo[k + 1] = h->R; list_hi[k + 1] = h->R + h->M;
  d_lists = (int64_t*)p->alloc(sizeof(int64_t) * 2 * n_lists, p->alloc_ctx, stream);
  d_bounds = (int64_t*)p->alloc(sizeof(int64_t) * bounds.size(), p->alloc_ctx, stream);
  if (!d_lists || !d_bounds) { st = SPTIR_ERR_ALLOC; goto fail; }
  RGMS_HIP(hipMemcpyAsync(d_lists, list_lo.data(), sizeof(int64_t) * n_lists, hipMemcpyHostToDevice, stream));
  RGMS_HIP(hipMemcpyAsync(d_lists + n_lists, list_hi.data(), sizeof(int64_t) * n_lists, hipMemcpyHostToDevice, stream));
  {
    const int n_searches = n_lists * (n_relations + 1);
    hipLaunchKernelGGL(k_relation_bounds, dim3((n_searches + 255) / 256), dim3(256), 0, stream, n_lists, n_relations,
                       p->n_rows, d_lists, d_lists + n_lists, h->row_ids, d_bounds);
  }
  RGMS_HIP(hipGetLastError());
  RGMS_HIP(hipMemcpyAsync(bounds.data(), d_bounds, sizeof(int64_t) * bounds.size(), hipMemcpyDeviceToHost, stream));
  RGMS_HIP(hipStreamSynchronize(stream));

  // ---- tiles: ELL buckets relation by relation, widest first (the longest-running tiles start first), then
  //      the remainder pieces
  for (int i = k; i >= 0; --i) {
    for (int32_t r = 0; r < n_relations; ++r) {
      const int64_t qa = bounds[(size_t)i * (n_relations + 1) + r], qb = bounds[(size_t)i * (n_relations + 1) + r + 1];
      for (int64_t q = qa; q < qb; q += 32) {
        RgmsTile tl;
        tl.slot0 = bucket_slot_ptr[i] + ((q - bucket_row_ptr[i]) << i);
        tl.row0 = (int32_t)q; tl.n_rows = (int32_t)std::min<int64_t>(32, qb - q); tl.log2w = i; tl.rel = r;
        tl.last_len = 0; tl.pad_ = 0;
        tiles.push_back(tl);
      }
    }
  }
  for (int32_t r = 0; r < n_relations; ++r) {
    const size_t o = (size_t)(k + 1) * (n_relations + 1);
    for (int64_t q = bounds[o + r]; q < bounds[o + r + 1]; ++q) {
      const int64_t m = q - h->R;
      const int64_t begin = rem_ptr[m], len = rem_ptr[m + 1] - begin;
      const int64_t n_seg = (len + 31) / 32;
      for (int64_t s0 = 0; s0 < n_seg; s0 += 32) {
        RgmsTile tl;
        tl.slot0 = h->S + begin + s0 * 32;
        tl.row0 = (int32_t)q; tl.n_rows = (int32_t)std::min<int64_t>(32, n_seg - s0); tl.log2w = -1; tl.rel = r;
        const int64_t covered = (s0 + tl.n_rows) * 32;
        tl.last_len = (int32_t)(covered <= len ? 32 : len - (covered - 32));
        tl.pad_ = 0;
        tiles.push_back(tl);
      }
    }
  }
  p->n_tiles = (int64_t)tiles.size();
  p->tiles = (RgmsTile*)p->alloc(sizeof(RgmsTile) * std::max<size_t>(tiles.size(), 1), p->alloc_ctx, stream);
  if (!p->tiles) { st = SPTIR_ERR_ALLOC; goto fail; }
  p->device_bytes += sizeof(RgmsTile) * std::max<size_t>(tiles.size(), 1);
  if (!tiles.empty())
    RGMS_HIP(hipMemcpyAsync(p->tiles, tiles.data(), sizeof(RgmsTile) * tiles.size(), hipMemcpyHostToDevice, stream));
  RGMS_HIP(hipStreamSynchronize(stream));
  p->free_(d_lists, p->alloc_ctx);
  p->free_(d_bounds, p->alloc_ctx);
  *out = p;
  return SPTIR_OK;

fail:
  (void)hipStreamSynchronize(stream);
  if (d_lists) p->free_(d_lists, p->alloc_ctx);
  if (d_bounds) p->free_(d_bounds, p->alloc_ctx);
  sptir_rgms_destroy(p);
  return st;
#undef RGMS_HIP
}

extern "C" sptir_status_t sptir_rgms(const sptir_rgms_t* p, const float* X, const float* W, float* Y, int32_t d_in,
                                     int32_t d_out, void* stream_) {
  if (!p || d_in < 1 || d_out < 1) return SPTIR_ERR_INVALID_ARG;
  if (p->n_rows == 0) return SPTIR_OK;
  if (!Y || (p->nnz > 0 && (!X || !W))) return SPTIR_ERR_INVALID_ARG;
  if ((d_in != 32 && d_in != 64 && d_in != 128) || d_out % 32 != 0 || (((uintptr_t)X) & 15) != 0)
    return SPTIR_ERR_UNSUPPORTED;
  hipStream_t stream = (hipStream_t)stream_;
  const int64_t y_elems = (int64_t)p->n_rows * d_out;
  hipLaunchKernelGGL(k_fill_zero, dim3((unsigned)std::min<int64_t>((y_elems + 255) / 256, 8192)), dim3(256), 0, stream,
                     Y, y_elems);
  if (p->n_tiles > 0) {
    RgmsArgs a;
    a.tiles = p->tiles; a.row_ids = p->hyb->row_ids; a.cols = p->hyb->cols; a.vals = p->hyb->vals;
    a.X = X; a.W = W; a.Y = Y; a.n_tiles = p->n_tiles; a.n_rows = p->n_rows; a.d_in = d_in; a.d_out = d_out;
    dim3 grid((unsigned)((p->n_tiles + kRgmsWaves - 1) / kRgmsWaves)), block(64 * kRgmsWaves);
    if (d_in == 32) hipLaunchKernelGGL(k_rgms<1>, grid, block, 0, stream, a);
    else if (d_in == 64) hipLaunchKernelGGL(k_rgms<2>, grid, block, 0, stream, a);
    else hipLaunchKernelGGL(k_rgms<4>, grid, block, 0, stream, a);
  }
  SPTIR_HIP(hipGetLastError());
  return SPTIR_OK;
}
