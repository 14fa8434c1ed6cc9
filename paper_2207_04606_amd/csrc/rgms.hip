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
//              The operator moves 128-byte rows at random addresses (rows of
//              X in, rows of Y out): about 3 TB/s on this chip, whatever the
//              order of the tiles and however many loads are in flight
//              (measured).  The optional workspace path stores the product
//              rows and sums them per row of Y in a fixed order: reproducible
//              bits for about 20 % more time (one more pass over the rows).
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
  // scatter through the workspace: row pos_of_row[q] of `partial` receives the product row of stacked row q
  const int32_t* pos_of_row;
  float* partial;
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

// The gather step of one tile, for rows of 2^LOG2W slots (a remainder tile takes LOG2W = 5 and masks the tail of
// its last segment).  Lane group g owns rows g, g + 8, g + 16, g + 24.  All column / value loads of the tile are
// issued before the first gather and every gather is independent of the others, so that the two memory
// round trips of a tile overlap inside the wavefront instead of repeating once per row.
template <int TIN, int LOG2W>
__device__ __forceinline__ void gather_tile(const RgmsArgs& a, const RgmsTile& tile, bool ell, int lane, float* z,
                                            int z_stride) {
  constexpr int kW = 1 << LOG2W;
  constexpr int kOct = kW >= 8 ? kW / 8 : 1;       // octets per row
  constexpr int kPer = kW >= 8 ? 8 : kW;           // slots per octet
  const int g = lane >> 3, fl = lane & 7;
  int col[4][kOct];
  float val[4][kOct];
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    const int row = m * 8 + g;
    const bool row_in = row < tile.n_rows;
    const int len = !row_in ? 0 : (ell || row < tile.n_rows - 1) ? kW : tile.last_len;
    const int64_t base = tile.slot0 + (int64_t)(row_in ? row : 0) * kW;
#pragma unroll
    for (int o = 0; o < kOct; ++o) {
      const int j = o * 8 + fl;
      const bool in = j < len;
      col[m][o] = a.cols[base + (in ? j : 0)];
      val[m][o] = in ? a.vals[base + j] : 0.f;
    }
  }
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    float4 acc[TIN];
#pragma unroll
    for (int q = 0; q < TIN; ++q) acc[q] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int o = 0; o < kOct; ++o) {
#pragma unroll
      for (int u = 0; u < kPer; ++u) {
        const int c = __shfl(col[m][o], g * 8 + u, 64);
        const float v = __shfl(val[m][o], g * 8 + u, 64);
        const float* xr = a.X + (size_t)c * (32 * TIN) + 4 * fl;
#pragma unroll
        for (int q = 0; q < TIN; ++q) {
          const float4 x = *reinterpret_cast<const float4*>(xr + 32 * q);
          acc[q].x = fmaf(v, x.x, acc[q].x); acc[q].y = fmaf(v, x.y, acc[q].y);
          acc[q].z = fmaf(v, x.z, acc[q].z); acc[q].w = fmaf(v, x.w, acc[q].w);
        }
      }
    }
    const int row = m * 8 + g;
#pragma unroll
    for (int q = 0; q < TIN; ++q) {
      float* zr = z + row * z_stride + 32 * q + 4 * fl;
      zr[0] = acc[q].x; zr[1] = acc[q].y; zr[2] = acc[q].z; zr[3] = acc[q].w;
    }
  }
}

// TIN float4 per lane cover d_in = 32 * TIN floats of a row of X.  TO_WORKSPACE: the product rows are stored to
// `partial` (plain stores; k_rgms_reduce sums them per row of Y) instead of added to Y with atomics.
// The matrix product and the scatter of one tile whose 32 x d_in block sits in z.
template <int TIN, bool TO_WORKSPACE>
__device__ __forceinline__ void multiply_and_scatter(const RgmsArgs& a, const RgmsTile& tile, int lane, const float* z,
                                                     int z_stride) {
  constexpr int kDin = 32 * TIN;
  const bool ell = tile.log2w >= 0;
  // the stacked row of every tile row -> its row of Y, or of the workspace (lanes 0..31 hold rows 0..31)
  int y_row_reg = 0;
  if (lane < tile.n_rows) {
    if constexpr (TO_WORKSPACE) {
      y_row_reg = a.pos_of_row[tile.row0 + lane];  // (only ELL tiles take this path)
    } else {
      const int stacked = a.row_ids[tile.row0 + (ell ? lane : 0)];
      y_row_reg = stacked - tile.rel * a.n_rows;
    }
  }
  const float* w_rel = a.W + (size_t)tile.rel * kDin * (size_t)a.d_out;
  const int mi = lane & 31, kh = lane >> 5;  // this lane's row of A / column of B, and which of the two k it holds
  for (int n0 = 0; n0 < a.d_out; n0 += 32) {  // 32 columns of Y at a time
    floatx16 d;
#pragma unroll
    for (int v = 0; v < 16; ++v) d[v] = 0.f;
#pragma unroll 4
    for (int kk = 0; kk < kDin / 2; ++kk) {
      const float av = z[mi * z_stride + 2 * kk + kh];                      // A[mi][2kk + kh]
      const float bv = w_rel[(size_t)(2 * kk + kh) * a.d_out + n0 + mi];    // B[2kk + kh][mi]
      d = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, d, 0, 0, 0);
    }
    // d[v] = D[8*(v/4) + 4*kh + v%4][mi]
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = 8 * (v >> 2) + 4 * kh + (v & 3);
      const int y_row = __shfl(y_row_reg, row, 64);
      if (row < tile.n_rows) {
        if constexpr (TO_WORKSPACE) a.partial[(size_t)y_row * a.d_out + n0 + mi] = d[v];
        else atomicAdd(a.Y + (size_t)y_row * a.d_out + n0 + mi, d[v]);
      }
    }
  }
}

// One tile per wavefront.  TIN float4 per lane cover d_in = 32 * TIN floats of a row of X.  TO_WORKSPACE: the
// product rows are stored to `partial` (k_rgms_reduce sums them per row of Y) instead of added to Y with atomics.
template <int TIN, bool TO_WORKSPACE>
__global__ __launch_bounds__(64 * kRgmsWaves) void k_rgms(RgmsArgs a) {
  constexpr int kZStride = 32 * TIN + 1;  // odd stride: the column reads of the matrix product hit 32 different banks
  __shared__ float z_all[kRgmsWaves][32 * kZStride];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int64_t t = (int64_t)blockIdx.x * kRgmsWaves + wave;
  if (t >= a.n_tiles) return;  // (no barriers below: the wavefronts of a workgroup are independent)
  const RgmsTile tile = a.tiles[t];
  float* z = z_all[wave];
  const bool ell = tile.log2w >= 0;
  switch (tile.log2w) {  // (the bucket width is the same for the whole wavefront)
    case 0: gather_tile<TIN, 0>(a, tile, ell, lane, z, kZStride); break;
    case 1: gather_tile<TIN, 1>(a, tile, ell, lane, z, kZStride); break;
    case 2: gather_tile<TIN, 2>(a, tile, ell, lane, z, kZStride); break;
    case 3: gather_tile<TIN, 3>(a, tile, ell, lane, z, kZStride); break;
    case 4: gather_tile<TIN, 4>(a, tile, ell, lane, z, kZStride); break;
    default: gather_tile<TIN, 5>(a, tile, ell, lane, z, kZStride); break;
  }
  multiply_and_scatter<TIN, TO_WORKSPACE>(a, tile, lane, z, kZStride);
}

// Row i of Y = sum of the rows node_ptr[i] .. node_ptr[i+1] of `partial`, in that order (the (relation, row)
// pairs of row i, relations ascending).  Eight lanes per four consecutive rows of Y (their partial rows are
// neighbours in memory, and four independent sums keep four loads in flight), 32 columns at a time.
constexpr int kReduceRows = 4;
__global__ __launch_bounds__(256) void k_rgms_reduce(int32_t n_rows, int32_t d_out, const int32_t* __restrict__ node_ptr,
                                                     const float* __restrict__ partial, float* Y) {
  const int64_t row0 = ((int64_t)blockIdx.x * 32 + (threadIdx.x >> 3)) * kReduceRows;
  if (row0 >= n_rows) return;
  const int fl = threadIdx.x & 7;
  int lo[kReduceRows], cnt[kReduceRows], longest = 0;
#pragma unroll
  for (int k = 0; k < kReduceRows; ++k) {
    const int64_t r = row0 + k < n_rows ? row0 + k : n_rows - 1;
    lo[k] = node_ptr[r];
    cnt[k] = row0 + k < n_rows ? node_ptr[r + 1] - lo[k] : 0;
    longest = max(longest, cnt[k]);
  }
  for (int c0 = 0; c0 < d_out; c0 += 32) {
    float4 acc[kReduceRows];
#pragma unroll
    for (int k = 0; k < kReduceRows; ++k) acc[k] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int t = 0; t < longest; ++t) {
#pragma unroll
      for (int k = 0; k < kReduceRows; ++k) {
        if (t < cnt[k]) {
          const float4 v = *reinterpret_cast<const float4*>(partial + (size_t)(lo[k] + t) * d_out + c0 + 4 * fl);
          acc[k].x += v.x; acc[k].y += v.y; acc[k].z += v.z; acc[k].w += v.w;
        }
      }
    }
#pragma unroll
    for (int k = 0; k < kReduceRows; ++k)
      if (row0 + k < n_rows) *reinterpret_cast<float4*>(Y + (size_t)(row0 + k) * d_out + c0 + 4 * fl) = acc[k];
  }
}

// mask[i * words + r / 64] bit r % 64: the pair (relation r, row i) has 1 .. max_len entries (it is an ELL row of
// the 3-D hyb); count[i] = number of such relations
__global__ void k_node_masks(int32_t n_rows, int32_t n_rel, int32_t words, int32_t max_len,
                             const int32_t* __restrict__ indptr, unsigned long long* mask, int32_t* count) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_rows) return;
  int total = 0;
  for (int w = 0; w < words; ++w) {
    unsigned long long m = 0;
    for (int b = 0; b < 64 && w * 64 + b < n_rel; ++b) {
      const int64_t row = (int64_t)(w * 64 + b) * n_rows + i;
      const int len = indptr[row + 1] - indptr[row];
      if (len >= 1 && len <= max_len) m |= 1ull << b;
    }
    mask[i * words + w] = m;
    total += __popcll(m);
  }
  count[i] = total;
}

// pos_of_row[q] for every ELL row q: first partial row of its row of Y + the number of that row's relations below its own
__global__ void k_pair_positions(int64_t n_ell_rows, int32_t n_rows, int32_t words, const int32_t* __restrict__ row_ids,
                                 const unsigned long long* __restrict__ mask, const int32_t* __restrict__ node_ptr,
                                 int32_t* pos_of_row) {
  const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (q >= n_ell_rows) return;
  const int stacked = row_ids[q];
  const int r = stacked / n_rows, i = stacked - r * n_rows;
  int rank = 0;
  for (int w = 0; w * 64 < r; ++w) {
    unsigned long long m = mask[(int64_t)i * words + w];
    if ((w + 1) * 64 > r) m &= (1ull << (r - w * 64)) - 1ull;
    rank += __popcll(m);
  }
  pos_of_row[q] = node_ptr[i] + rank;
}

}  // namespace
}  // namespace sptir

// The handle behind sptir_rgms_t.
struct sptir_rgms_handle {
  int32_t n_rel, n_rows, n_cols, k;
  int64_t nnz;
  sptir_hyb_t* hyb;  // hyb(1, k) of the stacked matrix (canonical arrays only)
  sptir::RgmsTile* tiles;  // the ELL tiles, then the remainder tiles
  int64_t n_tiles, n_ell_tiles;
  // scatter workspace (optional): one row of workspace_d_out floats per ELL row
  int32_t workspace_d_out;
  float* partial;
  int32_t* pos_of_row;   // [R]
  int32_t* node_ptr;     // [n_rows + 1]
  size_t device_bytes;
  sptir_alloc_fn alloc;
  sptir_free_fn free_;
  void* alloc_ctx;
};

using namespace sptir;

extern "C" sptir_status_t sptir_rgms_destroy(sptir_rgms_t* p) {
  if (!p) return SPTIR_OK;
  void* ptrs[] = {p->tiles, p->partial, p->pos_of_row, p->node_ptr};
  for (void* q : ptrs)
    if (q) p->free_(q, p->alloc_ctx);
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
  o.n_tiles = p->n_tiles; o.workspace_d_out = p->workspace_d_out; o.reserved = 0;
  o.device_bytes = (int64_t)p->device_bytes + hi.device_bytes;
  *out = o;
  return SPTIR_OK;
}

extern "C" sptir_status_t sptir_rgms_build(const sptir_csr_t* stacked, int32_t n_relations, int32_t max_bucket_log2,
                                           int32_t workspace_d_out, void* stream_, sptir_rgms_t** out) {
  if (!stacked || !out || n_relations < 1) return SPTIR_ERR_INVALID_ARG;
  if (workspace_d_out < 0 || workspace_d_out % 32 != 0) return SPTIR_ERR_INVALID_ARG;
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
  sptir_build_options_t opt = complete_options(nullptr);
  opt.no_spmm_plan = 1;
  sptir_status_t st = hyb_build_impl(stacked, 1, k, opt, stream_, &p->hyb);
  if (st != SPTIR_OK) { delete p; return st; }

  const sptir_hyb* h = p->hyb;
  const int n_lists = k + 2;  // the ELL buckets and the remainder
  std::vector<int64_t> bucket_row_ptr((size_t)k + 2), bucket_slot_ptr((size_t)k + 2), rem_ptr((size_t)h->M + 1);
  std::vector<int64_t> list_lo((size_t)n_lists), list_hi((size_t)n_lists), bounds((size_t)n_lists * (n_relations + 1));
  std::vector<RgmsTile> tiles;
  int64_t* d_lists = nullptr;
  int64_t* d_bounds = nullptr;
  unsigned long long* d_mask = nullptr;
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
  p->n_ell_tiles = (int64_t)tiles.size();
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
  if (workspace_d_out > 0 && h->R > 0) {
    // ---- where every ELL row's product row goes: the pairs of a row of Y side by side, relations ascending
    const int32_t words = (n_relations + 63) / 64;
    std::vector<int32_t> node_ptr((size_t)p->n_rows + 1, 0);
    d_mask = (unsigned long long*)p->alloc(sizeof(unsigned long long) * (size_t)p->n_rows * words, p->alloc_ctx, stream);
    p->node_ptr = (int32_t*)p->alloc(sizeof(int32_t) * ((size_t)p->n_rows + 1), p->alloc_ctx, stream);
    p->pos_of_row = (int32_t*)p->alloc(sizeof(int32_t) * (size_t)h->R, p->alloc_ctx, stream);
    p->partial = (float*)p->alloc(sizeof(float) * (size_t)h->R * workspace_d_out, p->alloc_ctx, stream);
    if (!d_mask || !p->node_ptr || !p->pos_of_row || !p->partial) { st = SPTIR_ERR_ALLOC; goto fail; }
    p->device_bytes += sizeof(int32_t) * ((size_t)p->n_rows + 1 + (size_t)h->R) +
                       sizeof(float) * (size_t)h->R * workspace_d_out;
    hipLaunchKernelGGL(k_node_masks, dim3((unsigned)((p->n_rows + 255) / 256)), dim3(256), 0, stream, p->n_rows,
                       n_relations, words, 1 << k, stacked->indptr, d_mask, p->node_ptr + 1);
    RGMS_HIP(hipGetLastError());
    RGMS_HIP(hipMemcpyAsync(node_ptr.data() + 1, p->node_ptr + 1, sizeof(int32_t) * (size_t)p->n_rows,
                            hipMemcpyDeviceToHost, stream));
    RGMS_HIP(hipStreamSynchronize(stream));
    for (int32_t i = 0; i < p->n_rows; ++i) node_ptr[(size_t)i + 1] += node_ptr[i];  // (ends at R < 2^31)
    RGMS_HIP(hipMemcpyAsync(p->node_ptr, node_ptr.data(), sizeof(int32_t) * node_ptr.size(), hipMemcpyHostToDevice,
                            stream));
    hipLaunchKernelGGL(k_pair_positions, dim3((unsigned)((h->R + 255) / 256)), dim3(256), 0, stream, (int64_t)h->R,
                       p->n_rows, words, h->row_ids, d_mask, p->node_ptr, p->pos_of_row);
    RGMS_HIP(hipGetLastError());
    RGMS_HIP(hipStreamSynchronize(stream));  // node_ptr (host) goes out of scope
    p->workspace_d_out = workspace_d_out;
  }
  RGMS_HIP(hipStreamSynchronize(stream));
  p->free_(d_lists, p->alloc_ctx);
  p->free_(d_bounds, p->alloc_ctx);
  if (d_mask) p->free_(d_mask, p->alloc_ctx);
  *out = p;
  return SPTIR_OK;

fail:
  (void)hipStreamSynchronize(stream);
  if (d_lists) p->free_(d_lists, p->alloc_ctx);
  if (d_bounds) p->free_(d_bounds, p->alloc_ctx);
  if (d_mask) p->free_(d_mask, p->alloc_ctx);
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
  RgmsArgs a;
  a.tiles = p->tiles; a.row_ids = p->hyb->row_ids; a.cols = p->hyb->cols; a.vals = p->hyb->vals;
  a.X = X; a.W = W; a.Y = Y; a.n_tiles = p->n_tiles; a.n_rows = p->n_rows; a.d_in = d_in; a.d_out = d_out;
  a.pos_of_row = p->pos_of_row; a.partial = p->partial;
  const dim3 block(64 * kRgmsWaves);
  auto launch = [&](bool to_workspace, int64_t first, int64_t n) {
    if (n <= 0) return;
    RgmsArgs b = a;
    b.tiles = p->tiles + first; b.n_tiles = n;
    const dim3 grid((unsigned)((n + kRgmsWaves - 1) / kRgmsWaves));
    if (to_workspace) {
      if (d_in == 32) hipLaunchKernelGGL((k_rgms<1, true>), grid, block, 0, stream, b);
      else if (d_in == 64) hipLaunchKernelGGL((k_rgms<2, true>), grid, block, 0, stream, b);
      else hipLaunchKernelGGL((k_rgms<4, true>), grid, block, 0, stream, b);
    } else {
      if (d_in == 32) hipLaunchKernelGGL((k_rgms<1, false>), grid, block, 0, stream, b);
      else if (d_in == 64) hipLaunchKernelGGL((k_rgms<2, false>), grid, block, 0, stream, b);
      else hipLaunchKernelGGL((k_rgms<4, false>), grid, block, 0, stream, b);
    }
  };
  if (p->partial && d_out <= p->workspace_d_out && (((uintptr_t)Y) & 15) == 0) {
    // product rows to the workspace, one pass that sums them into Y (every row of Y is written: no zero fill),
    // then the few remainder tiles on top with atomics
    launch(true, 0, p->n_ell_tiles);
    hipLaunchKernelGGL(k_rgms_reduce, dim3((unsigned)((p->n_rows + 32 * kReduceRows - 1) / (32 * kReduceRows))), dim3(256),
                       0, stream, p->n_rows, d_out, p->node_ptr, p->partial, Y);
    launch(false, p->n_ell_tiles, p->n_tiles - p->n_ell_tiles);
  } else {
    hipLaunchKernelGGL(k_fill_zero, dim3((unsigned)std::min<int64_t>((y_elems + 255) / 256, 8192)), dim3(256), 0,
                       stream, Y, y_elems);
    launch(false, 0, p->n_tiles);
  }
  SPTIR_HIP(hipGetLastError());
  return SPTIR_OK;
}
