// SpMM Y = A X on the hyb(c,k) decomposition (section 4.2.1 of arXiv
// 2207.04606), and the single-pass CSR variant the paper calls "no-hyb".
//
// Mapping (gfx950, wave64).  The feature dimension is cut into tiles of
// LG*VEC floats (32 floats = one 128-byte line of X by default).  A wavefront
// owns one work item (a run of up to item_slots stored slots of one ELL bucket
// or of one remainder piece) for one feature tile.  Its 64 lanes form 64/LG
// lane groups; a group covers the tile with VEC floats per lane, so one wave
// load instruction gathers 64/LG different rows of X, each as one contiguous
// 128-byte read.  The stored (column, value) pairs are read 64 at a time, one
// per lane, and handed to the groups by cross-lane reads; partial sums stay in
// registers and leave the wave once per ELL row through float atomic adds
// (different column partitions contribute to the same row of Y).
//
// Workgroup -> (item, tile): consecutive workgroup ids are dealt round-robin to
// the 8 XCDs, each with a private L2.  Tiles are therefore bound to
// blockIdx.x % 8 where the tile count allows it, so that an XCD's L2 only ever
// holds its own feature tile of the X slice of the column partition in flight.
#include "sptir_internal.h"

namespace sptir {
namespace {

constexpr int kWavesPerBlock = 4;
constexpr int kSpmmBlock = 64 * kWavesPerBlock;

template <int VEC> struct Vec;
template <> struct Vec<4> { using type = float4; };
template <> struct Vec<2> { using type = float2; };
template <> struct Vec<1> { using type = float; };

template <int VEC>
__device__ __forceinline__ void load_vec(float (&x)[VEC], const float* p) {
  typename Vec<VEC>::type v = *reinterpret_cast<const typename Vec<VEC>::type*>(p);
  if constexpr (VEC == 4) { x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w; }
  else if constexpr (VEC == 2) { x[0] = v.x; x[1] = v.y; }
  else { x[0] = v; }
}

enum TileMap : int {
  kMapTilesPerXcd = 0,  // n_tiles multiple of 8: XCD x owns tiles x, x+8, ...
  kMapXcdsPerTile = 1,  // n_tiles in {1,2,4}: 8/n_tiles XCDs share a tile, split the items
  kMapPlain = 2         // any other tile count: tile = id % n_tiles
};

struct SpmmArgs {
  const WorkItem* items;
  int64_t n_items;
  const int32_t* row_ids;
  const int32_t* cols;
  const float* vals;
  const float* X;
  float* Y;
  int32_t feat;
  int32_t n_tiles;
  int32_t map_mode;
  int32_t map_param;
};

// Walks `count` stored slots starting at cols/vals[slot0] for the feature
// offset f0 of this lane.  Slot o belongs to output row (row0 + (o >> lw)).
// DIRECT: the caller guarantees a single row that no other wave touches, so
// the result is stored instead of added, and row0 is the row of Y itself.
template <int VEC, int LG, bool DIRECT>
__device__ __forceinline__ void walk_item(const int32_t* __restrict__ cols, const float* __restrict__ vals,
                                          const int32_t* __restrict__ row_ids, const float* __restrict__ X,
                                          float* __restrict__ Y, int feat, int64_t slot0, int row0, int lw,
                                          int count, int lane, int f0, bool f_active) {
  constexpr int LOG2LG = (LG == 1) ? 0 : (LG == 2) ? 1 : (LG == 4) ? 2 : (LG == 8) ? 3 : (LG == 16) ? 4
                                     : (LG == 32) ? 5 : 6;
  constexpr int UB = LG < 8 ? LG : 8;  // gathers issued back to back before their FMAs
  const int group_base = lane & ~(LG - 1);
  const float* Xf = X + f0;
  float acc[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) acc[e] = 0.f;

  const int nch = (count + 63) >> 6;
  const int32_t* cp = cols + slot0;
  const float* vp = vals + slot0;
  int o = lane;
  int oc = o < count ? o : count - 1;
  int next_col = nch > 0 ? cp[oc] : 0;
  float next_val = (nch > 0 && o < count) ? vp[oc] : 0.f;

  for (int ch = 0; ch < nch; ++ch) {
    const int my_col = next_col;
    const float my_val = next_val;
    if (ch + 1 < nch) {  // fetch the next 64 (column, value) pairs early
      o = ((ch + 1) << 6) + lane;
      oc = o < count ? o : count - 1;
      next_col = cp[oc];
      next_val = o < count ? vp[oc] : 0.f;
    }
#pragma unroll
    for (int ub = 0; ub < LG; ub += UB) {
      float x[UB][VEC];
#pragma unroll
      for (int u = 0; u < UB; ++u) {
        int c = __shfl(my_col, group_base | (ub + u), 64);
        if (f_active) load_vec<VEC>(x[u], Xf + (size_t)c * (size_t)feat);
        else {
#pragma unroll
          for (int e = 0; e < VEC; ++e) x[u][e] = 0.f;
        }
      }
#pragma unroll
      for (int u = 0; u < UB; ++u) {
        float v = __shfl(my_val, group_base | (ub + u), 64);
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] = fmaf(v, x[u][e], acc[e]);
        if constexpr (!DIRECT) {
          // rows no wider than a lane group end inside the group: no cross-lane sum
          if (lw <= LOG2LG && (((ub + u + 1) & ((1 << lw) - 1)) == 0)) {
            int o_last = (ch << 6) + group_base + ub + u;
            if (f_active && o_last < count) {
              int r = row_ids[row0 + (o_last >> lw)];
              float* y = Y + (size_t)r * (size_t)feat + f0;
#pragma unroll
              for (int e = 0; e < VEC; ++e) unsafeAtomicAdd(y + e, acc[e]);
            }
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
          }
        }
      }
    }
    if (DIRECT || lw > LOG2LG) {
      // a wider row spans several lane groups (and, from 64 slots on, several chunks)
      bool row_done = (ch == nch - 1) || (!DIRECT && (lw < 6 || ((((unsigned)(ch + 1)) << 6) & ((1u << lw) - 1u)) == 0));
      if (row_done) {
        const int span = (DIRECT || lw >= 6) ? 64 : (1 << lw);  // lanes that share the row
        for (int d = LG; d < span; d <<= 1) {
#pragma unroll
          for (int e = 0; e < VEC; ++e) acc[e] += __shfl_xor(acc[e], d, 64);
        }
        int o_first = (ch << 6) + (lane & ~(span - 1));
        if (f_active && (lane & (span - 1)) < LG && (DIRECT || o_first < count)) {
          if constexpr (DIRECT) {
            float* y = Y + (size_t)row0 * (size_t)feat + f0;
#pragma unroll
            for (int e = 0; e < VEC; ++e) y[e] = acc[e];
          } else {
            int r = row_ids[row0 + (o_first >> lw)];
            float* y = Y + (size_t)r * (size_t)feat + f0;
#pragma unroll
            for (int e = 0; e < VEC; ++e) unsafeAtomicAdd(y + e, acc[e]);
          }
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
      }
    }
  }
  if constexpr (DIRECT) {
    if (nch == 0 && f_active && lane < LG) {  // empty row: Y row is zero
      float* y = Y + (size_t)row0 * (size_t)feat + f0;
#pragma unroll
      for (int e = 0; e < VEC; ++e) y[e] = 0.f;
    }
  }
}

// workgroup id -> (group of kWavesPerBlock consecutive units, feature tile)
__device__ __forceinline__ void decode_block(int map_mode, int map_param, int n_tiles, int64_t* group, int* tile) {
  unsigned bid = blockIdx.x;
  if (map_mode == kMapTilesPerXcd) {
    unsigned q = bid >> 3, x = bid & 7;
    *tile = (int)(x + 8 * (q % (unsigned)map_param));
    *group = q / (unsigned)map_param;
  } else if (map_mode == kMapXcdsPerTile) {
    unsigned q = bid >> 3, x = bid & 7;
    *tile = (int)(x % (unsigned)n_tiles);
    *group = (int64_t)q * map_param + x / (unsigned)n_tiles;
  } else {
    *tile = (int)(bid % (unsigned)n_tiles);
    *group = bid / (unsigned)n_tiles;
  }
}

template <int VEC, int LG>
__global__ __launch_bounds__(kSpmmBlock) void k_spmm_hyb(SpmmArgs a) {
  int64_t group;
  int tile;
  decode_block(a.map_mode, a.map_param, a.n_tiles, &group, &tile);
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int64_t item = group * kWavesPerBlock + wave;
  if (item >= a.n_items) return;
  const WorkItem it = a.items[item];
  const int lane = threadIdx.x & 63;
  const int f0 = tile * (LG * VEC) + (lane & (LG - 1)) * VEC;
  walk_item<VEC, LG, false>(a.cols, a.vals, a.row_ids, a.X, a.Y, a.feat, it.slot0, it.row0, (int)(it.meta & 63u),
                            (int)(it.meta >> 6), lane, f0, f0 < a.feat);
}

struct CsrArgs {
  const int32_t* indptr;
  const int32_t* indices;
  const float* values;
  const float* X;
  float* Y;
  int32_t n_rows;
  int32_t feat;
  int32_t n_tiles;
  int32_t map_mode;
  int32_t map_param;
};

// no-hyb: one wavefront per (row, feature tile); the row is walked whole
template <int VEC, int LG>
__global__ __launch_bounds__(kSpmmBlock) void k_spmm_csr(CsrArgs a) {
  int64_t group;
  int tile;
  decode_block(a.map_mode, a.map_param, a.n_tiles, &group, &tile);
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int64_t row = group * kWavesPerBlock + wave;
  if (row >= a.n_rows) return;
  const int begin = a.indptr[row], end = a.indptr[row + 1];
  const int lane = threadIdx.x & 63;
  const int f0 = tile * (LG * VEC) + (lane & (LG - 1)) * VEC;
  walk_item<VEC, LG, true>(a.indices, a.values, nullptr, a.X, a.Y, a.feat, begin, (int)row, kRemLog2W, end - begin,
                           lane, f0, f0 < a.feat);
}

__global__ void k_fill_zero_f4(float4* p, int64_t n4) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t step = (int64_t)gridDim.x * blockDim.x;
  for (; i < n4; i += step) p[i] = make_float4(0.f, 0.f, 0.f, 0.f);
}

__global__ void k_fill_zero_f1(float* p, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t step = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += step) p[i] = 0.f;
}

// launch geometry shared by both SpMM entry points
struct Geometry {
  int vec, lg, n_tiles, map_mode, map_param;
  int64_t grid;
};

bool plan(int64_t n_units, int feat, const void* X, const void* Y, Geometry* g) {
  uintptr_t align = (uintptr_t)X | (uintptr_t)Y;
  if (feat % 4 == 0 && (align & 15) == 0) { g->vec = 4; g->lg = feat <= 16 ? 4 : 8; }
  else if (feat % 2 == 0 && (align & 7) == 0) { g->vec = 2; g->lg = 16; }
  else { g->vec = 1; g->lg = 32; }
  int tf = g->vec * g->lg;
  g->n_tiles = (feat + tf - 1) / tf;
  int64_t groups = (n_units + kWavesPerBlock - 1) / kWavesPerBlock;
  if (g->n_tiles % 8 == 0) {
    g->map_mode = kMapTilesPerXcd; g->map_param = g->n_tiles / 8;
    g->grid = groups * g->n_tiles;
  } else if (8 % g->n_tiles == 0) {
    g->map_mode = kMapXcdsPerTile; g->map_param = 8 / g->n_tiles;
    g->grid = 8 * ((groups + g->map_param - 1) / g->map_param);
  } else {
    g->map_mode = kMapPlain; g->map_param = 0;
    g->grid = groups * g->n_tiles;
  }
  return g->grid <= 0x7FFFFFFF;
}

template <typename Args, typename K4_8, typename K4_4, typename K2, typename K1>
void launch_by_shape(const Geometry& g, hipStream_t stream, const Args& a, K4_8 k48, K4_4 k44, K2 k2, K1 k1) {
  dim3 grid((unsigned)g.grid), block(kSpmmBlock);
  if (g.vec == 4 && g.lg == 8) hipLaunchKernelGGL(k48, grid, block, 0, stream, a);
  else if (g.vec == 4) hipLaunchKernelGGL(k44, grid, block, 0, stream, a);
  else if (g.vec == 2) hipLaunchKernelGGL(k2, grid, block, 0, stream, a);
  else hipLaunchKernelGGL(k1, grid, block, 0, stream, a);
}

bool overlaps(const void* a, size_t na, const void* b, size_t nb) {
  uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
  return a0 < b0 + nb && b0 < a0 + na;
}

}  // namespace
}  // namespace sptir

using namespace sptir;

extern "C" sptir_status_t sptir_spmm(const sptir_hyb_t* h, const float* X, float* Y, int32_t feat, void* stream_) {
  if (!h || feat < 1) return SPTIR_ERR_INVALID_ARG;
  if ((h->n_cols > 0 && !X) || (h->n_rows > 0 && !Y)) return SPTIR_ERR_INVALID_ARG;
  const size_t x_bytes = sizeof(float) * (size_t)h->n_cols * feat, y_bytes = sizeof(float) * (size_t)h->n_rows * feat;
  if (x_bytes && y_bytes && overlaps(X, x_bytes, Y, y_bytes)) return SPTIR_ERR_INVALID_ARG;
  hipStream_t stream = (hipStream_t)stream_;
  if (h->n_rows == 0) return SPTIR_OK;

  // Y starts at zero (init block of the SpMM script, appendix A); a fill kernel
  // rather than a memset so that the call can be captured into a HIP graph
  const int64_t n_y = (int64_t)h->n_rows * feat;
  if (((uintptr_t)Y & 15) == 0 && n_y % 4 == 0) {
    int64_t n4 = n_y / 4;
    unsigned blocks = (unsigned)((n4 + 255) / 256 < 8192 ? (n4 + 255) / 256 : 8192);
    hipLaunchKernelGGL(k_fill_zero_f4, dim3(blocks), dim3(256), 0, stream, (float4*)Y, n4);
  } else {
    unsigned blocks = (unsigned)((n_y + 255) / 256 < 8192 ? (n_y + 255) / 256 : 8192);
    hipLaunchKernelGGL(k_fill_zero_f1, dim3(blocks), dim3(256), 0, stream, Y, n_y);
  }
  if (h->n_items > 0) {
    Geometry g;
    if (!plan(h->n_items, feat, X, Y, &g)) return SPTIR_ERR_OVERFLOW;
    SpmmArgs a;
    a.items = h->items; a.n_items = h->n_items; a.row_ids = h->row_ids; a.cols = h->cols; a.vals = h->vals;
    a.X = X; a.Y = Y; a.feat = feat; a.n_tiles = g.n_tiles; a.map_mode = g.map_mode; a.map_param = g.map_param;
    launch_by_shape(g, stream, a, k_spmm_hyb<4, 8>, k_spmm_hyb<4, 4>, k_spmm_hyb<2, 16>, k_spmm_hyb<1, 32>);
  }
  SPTIR_HIP(hipGetLastError());
  return SPTIR_OK;
}

extern "C" sptir_status_t sptir_spmm_csr(const sptir_csr_t* csr, const float* X, float* Y, int32_t feat,
                                         void* stream_) {
  if (!csr || feat < 1 || csr->n_rows < 0 || csr->n_cols < 0 || csr->nnz < 0) return SPTIR_ERR_INVALID_ARG;
  if (!csr->indptr || (csr->nnz > 0 && (!csr->indices || !csr->values))) return SPTIR_ERR_INVALID_ARG;
  if ((csr->n_cols > 0 && !X) || (csr->n_rows > 0 && !Y)) return SPTIR_ERR_INVALID_ARG;
  const size_t x_bytes = sizeof(float) * (size_t)csr->n_cols * feat, y_bytes = sizeof(float) * (size_t)csr->n_rows * feat;
  if (x_bytes && y_bytes && overlaps(X, x_bytes, Y, y_bytes)) return SPTIR_ERR_INVALID_ARG;
  if (csr->n_rows == 0) return SPTIR_OK;
  Geometry g;
  if (!plan(csr->n_rows, feat, X, Y, &g)) return SPTIR_ERR_OVERFLOW;
  CsrArgs a;
  a.indptr = csr->indptr; a.indices = csr->indices; a.values = csr->values; a.X = X; a.Y = Y;
  a.n_rows = csr->n_rows; a.feat = feat; a.n_tiles = g.n_tiles; a.map_mode = g.map_mode; a.map_param = g.map_param;
  launch_by_shape(g, (hipStream_t)stream_, a, k_spmm_csr<4, 8>, k_spmm_csr<4, 4>, k_spmm_csr<2, 16>,
                  k_spmm_csr<1, 32>);
  SPTIR_HIP(hipGetLastError());
  return SPTIR_OK;
}
