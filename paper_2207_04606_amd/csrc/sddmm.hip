// SDDMM on CSR: B[i,j] = A[i,j] * sum_k X[i,k] * Y[k,j] for the stored (i,j)
// of A (the SDDMM equation of section 4.2 of arXiv 2207.04606).  The paper
// runs SDDMM on plain CSR ("no composable formats"), iterates over the
// non-zeros directly (its sparse_fuse primitive) and reduces in two stages
// with vector loads; the mapping below keeps those three ideas.
//
// Mapping (gfx950, wave64).  The non-zeros are cut into runs of 64*kChunks
// consecutive entries, one wavefront each, so the work per wavefront is the
// same whatever the row lengths.  A wavefront takes 64 entries at a time with
// one coalesced load of their columns and values.  Eight lane groups of eight
// lanes then work on eight entries at once: lane fl of a group holds floats
// 4*(8t + fl) .. +3 (t = 0..T-1) of the entry's row of X in registers (loaded
// only when the row changes) and gathers the same floats of row j of Yt, one
// 128-byte line per group and load.  Stage one of the reduction is the lane's
// own dot product; stage two is a reduce-scatter over the eight lanes of the
// group, after which a lane transpose puts the 64 results back in entry order
// for one coalesced store.
#include "sptir_internal.h"

namespace sptir {
namespace {

constexpr int kSddmmWaves = 4;
constexpr int kSddmmChunks = 8;  // 64-entry chunks per wavefront
constexpr int kSddmmRun = 64 * kSddmmChunks;

struct SddmmArgs {
  const int32_t* indptr;
  const int32_t* indices;
  const float* values;
  const float* X;   // [n_rows, feat]
  const float* Yt;  // [n_cols, feat]
  float* B;         // [nnz]
  int64_t nnz;
  int32_t n_rows;
  int32_t feat;
};

// largest r in [0, n_rows) with indptr[r] <= e (e < nnz, so it exists)
__device__ __forceinline__ int row_of_entry(const int32_t* __restrict__ indptr, int n_rows, int64_t e) {
  int lo = 0, hi = n_rows;  // invariant: indptr[lo] <= e < indptr[hi]
  while (hi - lo > 1) {
    int mid = lo + ((hi - lo) >> 1);
    if ((int64_t)indptr[mid] <= e) lo = mid; else hi = mid;
  }
  return lo;
}

__device__ __forceinline__ float dot4(const float4& a, const float4& b, float acc) {
  acc = fmaf(a.x, b.x, acc);
  acc = fmaf(a.y, b.y, acc);
  acc = fmaf(a.z, b.z, acc);
  return fmaf(a.w, b.w, acc);
}

// Eight partial sums per lane -> lane fl of every 8-lane group ends with the group's total of p[fl].
__device__ __forceinline__ float reduce_scatter8(float (&p)[8], int fl) {
  float q[4], r[2];
  const bool hi4 = (fl & 4) != 0, hi2 = (fl & 2) != 0, hi1 = (fl & 1) != 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {  // partner fl^4 keeps the other half
    float keep = hi4 ? p[i + 4] : p[i], give = hi4 ? p[i] : p[i + 4];
    q[i] = keep + __shfl_xor(give, 4, 64);
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    float keep = hi2 ? q[i + 2] : q[i], give = hi2 ? q[i] : q[i + 2];
    r[i] = keep + __shfl_xor(give, 2, 64);
  }
  float keep = hi1 ? r[1] : r[0], give = hi1 ? r[0] : r[1];
  return keep + __shfl_xor(give, 1, 64);
}

// T float4 per lane cover feat <= 32*T floats; FULL: feat == 32*T, no lane is past the end
// (The second launch bound tells the register allocator how many wavefronts per SIMD to leave room for; left
//  alone it spreads the pipeline stages over 280+ registers although 16*T + 30 are live at any time.)
template <int T, bool FULL>
__global__ __launch_bounds__(64 * kSddmmWaves, T <= 4 ? 4 : 2) void k_sddmm(SddmmArgs a) {
  const int lane = threadIdx.x & 63, g = lane >> 3, fl = lane & 7;
  const int64_t run = (int64_t)blockIdx.x * kSddmmWaves + (threadIdx.x >> 6);
  const int64_t e_begin = run * kSddmmRun;
  if (e_begin >= a.nnz) return;
  const int64_t e_end = min(a.nnz, e_begin + kSddmmRun);
  const size_t feat = (size_t)a.feat;

  bool f_ok[T];
#pragma unroll
  for (int t = 0; t < T; ++t) f_ok[t] = FULL || 4 * (8 * t + fl) < a.feat;
  const int f_lane = 4 * fl;  // float offset of this lane inside every 32-float stripe

  int row_lo = row_of_entry(a.indptr, a.n_rows, e_begin);  // row of the chunk's first entry (wave-uniform)
  float4 x[T];
  int x_row = -1;
#pragma unroll
  for (int t = 0; t < T; ++t) x[t] = make_float4(0.f, 0.f, 0.f, 0.f);

  for (int64_t base = e_begin; base < e_end; base += 64) {
    const int64_t e_lane = base + lane;
    const bool in = e_lane < e_end;
    const int col_reg = in ? a.indices[e_lane] : 0;
    const float val_reg = in ? a.values[e_lane] : 0.f;
    // the row of this lane's entry: walk on from the chunk's first row
    int row_reg = row_lo;
    if (in) {
      while (row_reg + 1 < a.n_rows && e_lane >= (int64_t)a.indptr[row_reg + 1]) ++row_reg;
    }
    // Gathers run kAhead entries ahead of the multiplies; the scheduling barriers keep the compiler from
    // hoisting all eight entries' loads to the top (T*8 float4 of registers).
    constexpr int kAhead = T <= 8 ? 2 : 1;
    float4 y[kAhead + 1][T];
    auto issue = [&](int i, float4 (&yb)[T]) {
      const int c = __shfl(col_reg, i * 8 + g, 64);  // lane i*8+g fetched this group's i-th entry
      const float* yr = a.Yt + (size_t)c * feat + f_lane;
#pragma unroll
      for (int t = 0; t < T; ++t) {
        if (FULL || f_ok[t]) yb[t] = *reinterpret_cast<const float4*>(yr + 32 * t);
        else yb[t] = make_float4(0.f, 0.f, 0.f, 0.f);
      }
    };
    float p[8];
#pragma unroll
    for (int i = 0; i < kAhead; ++i) issue(i, y[i]);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int r = __shfl(row_reg, i * 8 + g, 64);
      if (r != x_row) {  // (entries past the end carry row_lo: a harmless reload)
        const float* xr = a.X + (size_t)r * feat + f_lane;
#pragma unroll
        for (int t = 0; t < T; ++t) {
          x[t] = f_ok[t] ? *reinterpret_cast<const float4*>(xr + 32 * t) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        x_row = r;
      }
      if (i + kAhead < 8) issue(i + kAhead, y[(i + kAhead) % (kAhead + 1)]);
      float acc = 0.f;
#pragma unroll
      for (int t = 0; t < T; ++t) acc = dot4(x[t], y[i % (kAhead + 1)][t], acc);
      // pin the multiplies here: left free, they are sunk to the use of p[] after the loop and every
      // gathered line stays live (and spills) until then
      asm volatile("" : "+v"(acc));
      p[i] = acc;
      __builtin_amdgcn_sched_barrier(0);
    }
    const float total = reduce_scatter8(p, fl);               // lane (g, fl): entry base + fl*8 + g
    const float mine = __shfl(total, (lane & 7) * 8 + (lane >> 3), 64);  // lane L: entry base + L
    if (in) a.B[e_lane] = val_reg * mine;
    row_lo = __builtin_amdgcn_readlane(row_reg, 63);  // (a lane past the end kept row_lo itself)
    // the last lane's entry may lie past the end only in the run's last chunk, after which nothing follows
  }
}

// Any feat and alignment: one entry at a time, the 64 lanes stride over the features.
__global__ __launch_bounds__(64 * kSddmmWaves) void k_sddmm_generic(SddmmArgs a) {
  const int lane = threadIdx.x & 63;
  const int64_t run = (int64_t)blockIdx.x * kSddmmWaves + (threadIdx.x >> 6);
  const int64_t e_begin = run * kSddmmRun;
  if (e_begin >= a.nnz) return;
  const int64_t e_end = min(a.nnz, e_begin + kSddmmRun);
  int row = row_of_entry(a.indptr, a.n_rows, e_begin);
  for (int64_t e = e_begin; e < e_end; ++e) {
    while (row + 1 < a.n_rows && e >= (int64_t)a.indptr[row + 1]) ++row;
    const float* xr = a.X + (size_t)row * (size_t)a.feat;
    const float* yr = a.Yt + (size_t)a.indices[e] * (size_t)a.feat;
    float acc = 0.f;
    for (int f = lane; f < a.feat; f += 64) acc = fmaf(xr[f], yr[f], acc);
    for (int d = 32; d > 0; d >>= 1) acc += __shfl_xor(acc, d, 64);
    if (lane == 0) a.B[e] = a.values[e] * acc;
  }
}

template <int T>
void launch_sddmm(const SddmmArgs& a, dim3 grid, hipStream_t stream) {
  if (a.feat == 32 * T) hipLaunchKernelGGL((k_sddmm<T, true>), grid, dim3(64 * kSddmmWaves), 0, stream, a);
  else hipLaunchKernelGGL((k_sddmm<T, false>), grid, dim3(64 * kSddmmWaves), 0, stream, a);
}

bool ranges_overlap(const void* a, size_t na, const void* b, size_t nb) {
  uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
  return na && nb && a0 < b0 + nb && b0 < a0 + na;
}

}  // namespace
}  // namespace sptir

using namespace sptir;

extern "C" sptir_status_t sptir_sddmm_csr(const sptir_csr_t* csr, const float* X, const float* Yt, float* B_values,
                                          int32_t feat, void* stream_) {
  if (!csr || feat < 1 || csr->n_rows < 0 || csr->n_cols < 0 || csr->nnz < 0) return SPTIR_ERR_INVALID_ARG;
  if (csr->nnz >= ((int64_t)1 << 31)) return SPTIR_ERR_OVERFLOW;
  if (csr->nnz == 0) return SPTIR_OK;
  if (!csr->indptr || !csr->indices || !csr->values || !X || !Yt || !B_values) return SPTIR_ERR_INVALID_ARG;
  if (csr->n_rows == 0 || csr->n_cols == 0) return SPTIR_ERR_INVALID_ARG;
  const size_t b_bytes = sizeof(float) * (size_t)csr->nnz;
  if (ranges_overlap(B_values, b_bytes, X, sizeof(float) * (size_t)csr->n_rows * feat) ||
      ranges_overlap(B_values, b_bytes, Yt, sizeof(float) * (size_t)csr->n_cols * feat) ||
      ranges_overlap(B_values, b_bytes, csr->indices, sizeof(int32_t) * (size_t)csr->nnz) ||
      ranges_overlap(B_values, b_bytes, csr->indptr, sizeof(int32_t) * ((size_t)csr->n_rows + 1)))
    return SPTIR_ERR_INVALID_ARG;
  SddmmArgs a;
  a.indptr = csr->indptr; a.indices = csr->indices; a.values = csr->values;
  a.X = X; a.Yt = Yt; a.B = B_values; a.nnz = csr->nnz; a.n_rows = csr->n_rows; a.feat = feat;
  const int64_t runs = (csr->nnz + kSddmmRun - 1) / kSddmmRun;
  dim3 grid((unsigned)((runs + kSddmmWaves - 1) / kSddmmWaves));
  hipStream_t stream = (hipStream_t)stream_;
  const bool vec4 = feat % 4 == 0 && ((((uintptr_t)X) | ((uintptr_t)Yt)) & 15) == 0;
  if (!vec4 || feat > 512) hipLaunchKernelGGL(k_sddmm_generic, grid, dim3(64 * kSddmmWaves), 0, stream, a);
  else if (feat <= 32) launch_sddmm<1>(a, grid, stream);
  else if (feat <= 64) launch_sddmm<2>(a, grid, stream);
  else if (feat <= 128) launch_sddmm<4>(a, grid, stream);
  else if (feat <= 256) launch_sddmm<8>(a, grid, stream);
  else launch_sddmm<16>(a, grid, stream);
  SPTIR_HIP(hipGetLastError());
  return SPTIR_OK;
}
