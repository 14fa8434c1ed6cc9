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
// lanes then work on eight entries at once (group g on entries 8g .. 8g+7 of
// the 64, one after the other, so that its row changes rarely): lane fl of a group holds floats
// 4*(8t + fl) .. +3 (t = 0..T-1) of the entry's row of X in registers (loaded
// only when the row changes) and gathers the same floats of row j of Yt, one
// 128-byte line per group and load.  Stage one of the reduction is the lane's
// own dot product; stage two is a reduce-scatter over the eight lanes of the
// group, which leaves lane 8g + fl with the result of entry 8g + fl: the 64
// results are in entry order for one coalesced store.
//
// With a plan (sptir_sddmm_plan_build) the entries are visited in column-
// partition order instead of CSR order, the locality argument section 4.2.1
// makes for SpMM applied to SDDMM: the plan lists the entries of partition p
// (rows ascending) as (row, column, CSR position) triples, every XCD is given
// its own partitions, and the workgroups of an XCD sweep them one after the
// other, so an XCD's L2 holds the rows of Yt of one partition at a time.
// There is nothing to accumulate across partitions - an entry's result is
// complete where it is computed - so one launch covers all of them.
#include <string.h>

#include <algorithm>
#include <new>
#include <vector>

#include "sptir_internal.h"
#include "sptir_scan.h"

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
  // with a plan: entries in partition order, and where each XCD's runs start
  const int32_t* e_row;
  const int32_t* e_col;
  const int32_t* e_pos;
  const int64_t* run_first_entry;  // [n_runs]: first entry of every run (at most kSddmmRun entries of one
  const int32_t* run_len;          //           partition, run_len of them), runs grouped by XCD
  const int32_t* xcd_run_ptr;      // [9]: the runs of XCD x are xcd_run_ptr[x] .. xcd_run_ptr[x+1]
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
template <int T, bool FULL, bool PLAN>
__global__ __launch_bounds__(64 * kSddmmWaves, T <= 4 ? 4 : 2) void k_sddmm(SddmmArgs a) {
  const int lane = threadIdx.x & 63, g = lane >> 3, fl = lane & 7;
  int64_t e_begin, e_end;
  if constexpr (PLAN) {
    // consecutive workgroup ids go to consecutive XCDs: workgroup (x + 8*j) is the j-th of XCD x
    const int xcd = blockIdx.x & 7;
    const int64_t run = (int64_t)a.xcd_run_ptr[xcd] + (int64_t)(blockIdx.x >> 3) * kSddmmWaves + (threadIdx.x >> 6);
    if (run >= a.xcd_run_ptr[xcd + 1]) return;
    e_begin = a.run_first_entry[run];
    e_end = e_begin + a.run_len[run];
  } else {
    const int64_t run = (int64_t)blockIdx.x * kSddmmWaves + (threadIdx.x >> 6);
    e_begin = run * kSddmmRun;
    if (e_begin >= a.nnz) return;
    e_end = min(a.nnz, e_begin + kSddmmRun);
  }
  const size_t feat = (size_t)a.feat;

  bool f_ok[T];
#pragma unroll
  for (int t = 0; t < T; ++t) f_ok[t] = FULL || 4 * (8 * t + fl) < a.feat;
  const int f_lane = 4 * fl;  // float offset of this lane inside every 32-float stripe

  int row_lo = PLAN ? 0 : row_of_entry(a.indptr, a.n_rows, e_begin);  // row of the chunk's first entry (wave-uniform)
  // The rows of X a chunk needs are staged in LDS once per chunk: every load instruction then brings up to eight
  // different rows (one per lane group), where a reload inside the entry loop costs the address path a whole
  // instruction even if a single lane group asks for it - and in partition order a row lasts only a few entries.
  // (Measured: pays for feature sizes of 128 and 256 in partition order, costs a little everywhere else.)
  constexpr int kStage = !PLAN ? 0 : (T == 4 ? 16 : (T == 8 ? 8 : 0));  // rows of X staged per wavefront (8 KB)
  __shared__ __align__(16) float x_stage[kSddmmWaves][kStage > 0 ? kStage : 1][32 * T];
  __shared__ int row_table[kSddmmWaves][kStage > 0 ? kStage : 1];
  const int wave = threadIdx.x >> 6;
  float4 x[T];
  int x_row = -1;
#pragma unroll
  for (int t = 0; t < T; ++t) x[t] = make_float4(0.f, 0.f, 0.f, 0.f);

  for (int64_t base = e_begin; base < e_end; base += 64) {
    const int64_t e_lane = base + lane;
    const bool in = e_lane < e_end;
    int col_reg, row_reg;
    int64_t out_pos;
    float val_reg;
    if constexpr (PLAN) {
      const int64_t el = in ? e_lane : e_begin;  // (a lane past the end repeats the run's first entry)
      col_reg = a.e_col[el];
      row_reg = a.e_row[el];
      out_pos = a.e_pos[el];
      val_reg = a.values[out_pos];
    } else {
      col_reg = in ? a.indices[e_lane] : 0;
      val_reg = in ? a.values[e_lane] : 0.f;
      out_pos = e_lane;
      // the row of this lane's entry: walk on from the chunk's first row
      row_reg = row_lo;
      if (in) {
        while (row_reg + 1 < a.n_rows && e_lane >= (int64_t)a.indptr[row_reg + 1]) ++row_reg;
      }
    }
    bool staged = false;
    int rank_reg = 0, x_rank = -1;
    if constexpr (kStage > 0) {
      // entries arrive row by row: a lane whose row differs from its left neighbour's starts a new row
      const int left = __shfl_up(row_reg, 1, 64);
      const bool head = lane == 0 || row_reg != left;
      const unsigned long long heads = __ballot(head);
      const int n_distinct = __popcll(heads);
      rank_reg = __popcll(heads & ((2ull << lane) - 1ull)) - 1;  // which of the chunk's rows this lane's entry uses
      staged = n_distinct <= kStage;                             // (wave-uniform)
      if (staged) {
        if (head) row_table[wave][rank_reg] = row_reg;
        for (int k0 = 0; k0 < n_distinct; k0 += 8) {
          const int k = k0 + g;
          if (k < n_distinct) {
            const float* xr = a.X + (size_t)row_table[wave][k] * feat + f_lane;
#pragma unroll
            for (int t = 0; t < T; ++t) {
              const float4 v = f_ok[t] ? *reinterpret_cast<const float4*>(xr + 32 * t) : make_float4(0.f, 0.f, 0.f, 0.f);
              *reinterpret_cast<float4*>(&x_stage[wave][k][32 * t + f_lane]) = v;
            }
          }
        }
        x_row = -1;  // the registers are about to hold staged rows
      }
    }
    // Gathers run kAhead entries ahead of the multiplies; the scheduling barriers keep the compiler from
    // hoisting all eight entries' loads to the top (T*8 float4 of registers).
    constexpr int kAhead = T <= 8 ? 2 : 1;
    float4 y[kAhead + 1][T];
    auto issue = [&](int i, float4 (&yb)[T]) {
      const int c = __shfl(col_reg, g * 8 + i, 64);  // lane g*8+i fetched this group's i-th entry
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
      if (staged) {
        const int rk = __shfl(rank_reg, g * 8 + i, 64);
        if (rk != x_rank) {
#pragma unroll
          for (int t = 0; t < T; ++t) x[t] = *reinterpret_cast<const float4*>(&x_stage[wave][rk][32 * t + f_lane]);
          x_rank = rk;
        }
      } else {
        const int r = __shfl(row_reg, g * 8 + i, 64);
        if (r != x_row) {  // (entries past the end carry a valid row: a harmless reload)
          const float* xr = a.X + (size_t)r * feat + f_lane;
#pragma unroll
          for (int t = 0; t < T; ++t) {
            x[t] = f_ok[t] ? *reinterpret_cast<const float4*>(xr + 32 * t) : make_float4(0.f, 0.f, 0.f, 0.f);
          }
          x_row = r;
        }
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
    // lane (g, fl) ends with the total of p[fl], i.e. of entry base + g*8 + fl = base + lane: its own entry
    const float mine = reduce_scatter8(p, fl);
    if (in) a.B[out_pos] = val_reg * mine;
    if constexpr (!PLAN) row_lo = __builtin_amdgcn_readlane(row_reg, 63);  // (a lane past the end kept row_lo itself)
    // the last lane's entry may lie past the end only in the run's last chunk, after which nothing follows
  }
}

// Any feat and alignment: one entry at a time, the 64 lanes stride over the features.
template <bool PLAN>
__global__ __launch_bounds__(64 * kSddmmWaves) void k_sddmm_generic(SddmmArgs a) {
  const int lane = threadIdx.x & 63;
  int64_t e_begin, e_end;
  if constexpr (PLAN) {
    const int xcd = blockIdx.x & 7;
    const int64_t run = (int64_t)a.xcd_run_ptr[xcd] + (int64_t)(blockIdx.x >> 3) * kSddmmWaves + (threadIdx.x >> 6);
    if (run >= a.xcd_run_ptr[xcd + 1]) return;
    e_begin = a.run_first_entry[run];
    e_end = e_begin + a.run_len[run];
  } else {
    const int64_t run = (int64_t)blockIdx.x * kSddmmWaves + (threadIdx.x >> 6);
    e_begin = run * kSddmmRun;
    if (e_begin >= a.nnz) return;
    e_end = min(a.nnz, e_begin + kSddmmRun);
  }
  int row = PLAN ? 0 : row_of_entry(a.indptr, a.n_rows, e_begin);
  for (int64_t e = e_begin; e < e_end; ++e) {
    int col;
    int64_t pos;
    if constexpr (PLAN) {
      row = a.e_row[e]; col = a.e_col[e]; pos = a.e_pos[e];
    } else {
      while (row + 1 < a.n_rows && e >= (int64_t)a.indptr[row + 1]) ++row;
      col = a.indices[e]; pos = e;
    }
    const float* xr = a.X + (size_t)row * (size_t)a.feat;
    const float* yr = a.Yt + (size_t)col * (size_t)a.feat;
    float acc = 0.f;
    for (int f = lane; f < a.feat; f += 64) acc = fmaf(xr[f], yr[f], acc);
    for (int d = 32; d > 0; d >>= 1) acc += __shfl_xor(acc, d, 64);
    if (lane == 0) a.B[pos] = a.values[pos] * acc;
  }
}

template <int T, bool PLAN>
void launch_sddmm(const SddmmArgs& a, dim3 grid, hipStream_t stream) {
  if (a.feat == 32 * T) hipLaunchKernelGGL((k_sddmm<T, true, PLAN>), grid, dim3(64 * kSddmmWaves), 0, stream, a);
  else hipLaunchKernelGGL((k_sddmm<T, false, PLAN>), grid, dim3(64 * kSddmmWaves), 0, stream, a);
}

template <bool PLAN>
void launch_sddmm_for_feat(const SddmmArgs& a, dim3 grid, hipStream_t stream) {
  if (a.feat <= 32) launch_sddmm<1, PLAN>(a, grid, stream);
  else if (a.feat <= 64) launch_sddmm<2, PLAN>(a, grid, stream);
  else if (a.feat <= 128) launch_sddmm<4, PLAN>(a, grid, stream);
  else if (a.feat <= 256) launch_sddmm<8, PLAN>(a, grid, stream);
  else launch_sddmm<16, PLAN>(a, grid, stream);
}

bool vector_path_ok(const float* X, const float* Yt, int32_t feat) {
  return feat % 4 == 0 && feat <= 512 && ((((uintptr_t)X) | ((uintptr_t)Yt)) & 15) == 0;
}

// ------------------------------------------------------------------- plan
// lens[p * n_rows + r] = entries of row r in column partition p
__global__ void k_piece_lengths(int32_t n_rows, int32_t c, int32_t w, const int32_t* __restrict__ indptr,
                                const int32_t* __restrict__ indices, int32_t* lens) {
  int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= (int64_t)n_rows * c) return;
  int r = (int)(t % n_rows), p = (int)(t / n_rows);
  int a = indptr[r], b = indptr[r + 1];
  int first = (p == 0) ? a : lower_bound_col(indices, a, b, (int64_t)p * w);
  int last = (p == c - 1) ? b : lower_bound_col(indices, first, b, (int64_t)(p + 1) * w);
  lens[t] = last - first;
}

// Copies every (row, partition) piece to its place in the partition-ordered entry list:
// offs[p * n_rows + r] is the piece's offset inside partition p, part_first[p] the partition's first entry.
__global__ void k_scatter_entries(int32_t n_rows, int32_t c, int32_t w, const int32_t* __restrict__ indptr,
                                  const int32_t* __restrict__ indices, const int32_t* __restrict__ offs,
                                  const int64_t* __restrict__ part_first, int32_t* e_row, int32_t* e_col,
                                  int32_t* e_pos) {
  int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= (int64_t)n_rows * c) return;
  int r = (int)(t % n_rows), p = (int)(t / n_rows);
  int a = indptr[r], b = indptr[r + 1];
  int first = (p == 0) ? a : lower_bound_col(indices, a, b, (int64_t)p * w);
  int last = (p == c - 1) ? b : lower_bound_col(indices, first, b, (int64_t)(p + 1) * w);
  int64_t dst = part_first[p] + offs[t];
  for (int q = first; q < last; ++q, ++dst) {
    e_row[dst] = r;
    e_col[dst] = indices[q];
    e_pos[dst] = q;
  }
}

bool ranges_overlap(const void* a, size_t na, const void* b, size_t nb) {
  uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
  return na && nb && a0 < b0 + nb && b0 < a0 + na;
}

}  // namespace
}  // namespace sptir

// The handle behind sptir_sddmm_plan_t.
struct sptir_sddmm_plan {
  int32_t n_rows, n_cols, c, w;
  int64_t nnz;
  // c >= 2: the entries in partition order and the runs of every XCD
  int32_t *e_row, *e_col, *e_pos;
  int64_t* run_first_entry;
  int32_t* run_len;
  int32_t* xcd_run_ptr;
  int64_t n_runs;
  int64_t max_runs_per_xcd;
  // c == 1: entries stay in CSR order; the plan keeps its own copy of the structure
  int32_t *indptr, *indices;
  size_t device_bytes;
  sptir_alloc_fn alloc;
  sptir_free_fn free_;
  void* alloc_ctx;
};

using namespace sptir;

extern "C" sptir_status_t sptir_sddmm_plan_destroy(sptir_sddmm_plan_t* p) {
  if (!p) return SPTIR_OK;
  void* ptrs[] = {p->e_row, p->e_col, p->e_pos, p->run_first_entry, p->run_len, p->xcd_run_ptr, p->indptr, p->indices};
  for (void* q : ptrs)
    if (q) p->free_(q, p->alloc_ctx);
  delete p;
  return SPTIR_OK;
}

extern "C" sptir_status_t sptir_sddmm_plan_info(const sptir_sddmm_plan_t* p, sptir_sddmm_plan_info_t* out) {
  if (!p || !out) return SPTIR_ERR_INVALID_ARG;
  sptir_sddmm_plan_info_t o;
  o.n_rows = p->n_rows; o.n_cols = p->n_cols; o.n_col_parts = p->c; o.part_width = p->w;
  o.nnz = p->nnz; o.n_runs = p->n_runs; o.device_bytes = (int64_t)p->device_bytes;
  *out = o;
  return SPTIR_OK;
}

extern "C" int32_t sptir_sddmm_default_col_parts(int32_t n_rows, int32_t n_cols, int64_t nnz, int32_t feat_hint) {
  // The rows of Yt of one partition should fit an XCD's L2 next to the rest of the traffic (2.5 of 4 MB); every
  // (row, partition) piece re-reads its row of X, so a piece should hold a few entries; every XCD wants its
  // own partitions, so c is a multiple of 8 - or 1, which leaves the entries in CSR order.
  if (n_rows <= 0 || n_cols <= 0 || nnz <= 0) return 1;
  const int64_t feat = feat_hint > 0 ? feat_hint : 128;
  const int64_t w_fit = std::max<int64_t>(1, (int64_t)(2.5 * 1024 * 1024) / (feat * 4));
  int64_t want = (n_cols + w_fit - 1) / w_fit;
  const int64_t by_piece = nnz / ((int64_t)n_rows * 4);
  // (to the nearest multiple of 8, as far as the pieces allow: measured, 7 wanted runs best with 8, 12 with 8)
  want = std::min((want + 3) / 8 * 8, by_piece / 8 * 8);
  return (want >= 8 && n_cols > w_fit) ? (int32_t)std::min<int64_t>(want, 1024) : 1;
}

extern "C" sptir_status_t sptir_sddmm_plan_build(const sptir_csr_t* csr, int32_t n_col_parts, int32_t feat_hint,
                                                 void* stream_, sptir_sddmm_plan_t** out) {
  if (!csr || !out || n_col_parts < 0 || feat_hint < 0) return SPTIR_ERR_INVALID_ARG;
  if (csr->n_rows < 0 || csr->n_cols < 0 || csr->nnz < 0) return SPTIR_ERR_INVALID_ARG;
  if (csr->nnz >= ((int64_t)1 << 31)) return SPTIR_ERR_OVERFLOW;
  if (!csr->indptr || (csr->nnz > 0 && !csr->indices)) return SPTIR_ERR_INVALID_ARG;
  if (csr->nnz > 0 && (csr->n_rows == 0 || csr->n_cols == 0)) return SPTIR_ERR_INVALID_ARG;
  hipStream_t stream = (hipStream_t)stream_;
  const int32_t n_rows = csr->n_rows, n_cols = csr->n_cols;
  const int64_t nnz = csr->nnz;

  // ---- number of column partitions
  int32_t c = n_col_parts > 0 ? n_col_parts : sptir_sddmm_default_col_parts(n_rows, n_cols, nnz, feat_hint);
  if (c > std::max(n_cols, 1)) c = std::max(n_cols, 1);
  if ((int64_t)n_rows * c > ((int64_t)1 << 36)) return SPTIR_ERR_OVERFLOW;

  sptir_sddmm_plan* p = new (std::nothrow) sptir_sddmm_plan();
  if (!p) return SPTIR_ERR_ALLOC;
  memset(p, 0, sizeof(*p));
  current_allocator(&p->alloc, &p->free_, &p->alloc_ctx);
  p->n_rows = n_rows; p->n_cols = n_cols; p->c = c; p->nnz = nnz;
  p->w = (int32_t)(((int64_t)n_cols + c - 1) / c);
  sptir_alloc_fn alloc = p->alloc; sptir_free_fn free_ = p->free_; void* actx = p->alloc_ctx;
  int32_t* lens = nullptr;
  int32_t* d_totals = nullptr;
  int64_t* d_part_first = nullptr;
  sptir_status_t st = SPTIR_OK;
  auto take = [&](void** dst, size_t bytes) {
    *dst = alloc(bytes ? bytes : 16, actx, stream);
    if (*dst) p->device_bytes += bytes ? bytes : 16;
    return *dst != nullptr;
  };
#define PLAN_HIP(call)                                                 \
  do {                                                                 \
    hipError_t e_ = (call);                                            \
    if (e_ != hipSuccess) { st = note_hip_error(e_, #call); goto fail; } \
  } while (0)

  if (c == 1 || nnz == 0) {
    p->c = 1; p->w = n_cols;
    if (!take((void**)&p->indptr, sizeof(int32_t) * ((size_t)n_rows + 1)) ||
        !take((void**)&p->indices, sizeof(int32_t) * (size_t)nnz)) { st = SPTIR_ERR_ALLOC; goto fail; }
    PLAN_HIP(hipMemcpyAsync(p->indptr, csr->indptr, sizeof(int32_t) * ((size_t)n_rows + 1), hipMemcpyDeviceToDevice,
                            stream));
    if (nnz > 0)
      PLAN_HIP(hipMemcpyAsync(p->indices, csr->indices, sizeof(int32_t) * (size_t)nnz, hipMemcpyDeviceToDevice,
                              stream));
    PLAN_HIP(hipStreamSynchronize(stream));
    *out = p;
    return SPTIR_OK;
  }
  {
    const int64_t n_pairs = (int64_t)n_rows * c;
    lens = (int32_t*)alloc(sizeof(int32_t) * (size_t)n_pairs, actx, stream);
    d_totals = (int32_t*)alloc(sizeof(int32_t) * (size_t)c, actx, stream);
    d_part_first = (int64_t*)alloc(sizeof(int64_t) * (size_t)c, actx, stream);
    if (!lens || !d_totals || !d_part_first) { st = SPTIR_ERR_ALLOC; goto fail; }
    const unsigned pair_blocks = (unsigned)((n_pairs + 255) / 256);
    hipLaunchKernelGGL(k_piece_lengths, dim3(pair_blocks), dim3(256), 0, stream, n_rows, c, p->w, csr->indptr,
                       csr->indices, lens);
    hipLaunchKernelGGL(k_scan_sequences<int32_t>, dim3((unsigned)c), dim3(kBuildBlock), 0, stream, lens, n_rows,
                       d_totals);
    PLAN_HIP(hipGetLastError());
    std::vector<int32_t> totals((size_t)c);
    PLAN_HIP(hipMemcpyAsync(totals.data(), d_totals, sizeof(int32_t) * (size_t)c, hipMemcpyDeviceToHost, stream));
    PLAN_HIP(hipStreamSynchronize(stream));
    std::vector<int64_t> part_first((size_t)c + 1, 0);
    for (int32_t q = 0; q < c; ++q) {
      if (totals[q] < 0) { st = SPTIR_ERR_UNSORTED; goto fail; }
      part_first[q + 1] = part_first[q] + totals[q];
    }
    // the pieces tile every row exactly when its columns ascend; anything else would not fit the arrays below
    if (part_first[c] != nnz) { st = SPTIR_ERR_UNSORTED; goto fail; }
    if (!take((void**)&p->e_row, sizeof(int32_t) * (size_t)nnz) || !take((void**)&p->e_col, sizeof(int32_t) * (size_t)nnz) ||
        !take((void**)&p->e_pos, sizeof(int32_t) * (size_t)nnz)) { st = SPTIR_ERR_ALLOC; goto fail; }
    PLAN_HIP(hipMemcpyAsync(d_part_first, part_first.data(), sizeof(int64_t) * (size_t)c, hipMemcpyHostToDevice,
                            stream));
    hipLaunchKernelGGL(k_scatter_entries, dim3(pair_blocks), dim3(256), 0, stream, n_rows, c, p->w, csr->indptr,
                       csr->indices, lens, d_part_first, p->e_row, p->e_col, p->e_pos);
    PLAN_HIP(hipGetLastError());

    // ---- partitions to XCDs (largest first onto the least loaded), runs of every XCD in partition order
    std::vector<int32_t> order((size_t)c);
    for (int32_t q = 0; q < c; ++q) order[q] = q;
    std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) { return totals[x] > totals[y]; });
    int64_t load[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    std::vector<int32_t> of_xcd[8];
    for (int32_t q : order) {
      int best = 0;
      for (int x = 1; x < 8; ++x)
        if (load[x] < load[best]) best = x;
      load[best] += totals[q];
      of_xcd[best].push_back(q);
    }
    std::vector<int64_t> run_first;
    std::vector<int32_t> run_len;
    int32_t xcd_run_ptr[9];
    int64_t max_runs = 0;
    for (int x = 0; x < 8; ++x) {
      xcd_run_ptr[x] = (int32_t)run_first.size();
      std::sort(of_xcd[x].begin(), of_xcd[x].end());
      for (int32_t q : of_xcd[x]) {
        for (int64_t off = 0; off < totals[q]; off += kSddmmRun) {
          run_first.push_back(part_first[q] + off);
          run_len.push_back((int32_t)std::min<int64_t>(kSddmmRun, totals[q] - off));
        }
      }
      max_runs = std::max<int64_t>(max_runs, (int64_t)run_first.size() - xcd_run_ptr[x]);
    }
    xcd_run_ptr[8] = (int32_t)run_first.size();
    p->n_runs = (int64_t)run_first.size();
    p->max_runs_per_xcd = max_runs;
    if (!take((void**)&p->run_first_entry, sizeof(int64_t) * run_first.size()) ||
        !take((void**)&p->run_len, sizeof(int32_t) * run_len.size()) ||
        !take((void**)&p->xcd_run_ptr, sizeof(xcd_run_ptr))) { st = SPTIR_ERR_ALLOC; goto fail; }
    PLAN_HIP(hipMemcpyAsync(p->run_first_entry, run_first.data(), sizeof(int64_t) * run_first.size(),
                            hipMemcpyHostToDevice, stream));
    PLAN_HIP(hipMemcpyAsync(p->run_len, run_len.data(), sizeof(int32_t) * run_len.size(), hipMemcpyHostToDevice,
                            stream));
    PLAN_HIP(hipMemcpyAsync(p->xcd_run_ptr, xcd_run_ptr, sizeof(xcd_run_ptr), hipMemcpyHostToDevice, stream));
    PLAN_HIP(hipStreamSynchronize(stream));  // the host vectors go out of scope
  }
  free_(lens, actx); free_(d_totals, actx); free_(d_part_first, actx);
  *out = p;
  return SPTIR_OK;

fail:
  (void)hipStreamSynchronize(stream);
  if (lens) free_(lens, actx);
  if (d_totals) free_(d_totals, actx);
  if (d_part_first) free_(d_part_first, actx);
  sptir_sddmm_plan_destroy(p);
  return st;
#undef PLAN_HIP
}

extern "C" sptir_status_t sptir_sddmm(const sptir_sddmm_plan_t* p, const float* values, const float* X,
                                      const float* Yt, float* B_values, int32_t feat, void* stream_) {
  if (!p || feat < 1) return SPTIR_ERR_INVALID_ARG;
  if (p->nnz == 0) return SPTIR_OK;
  if (!values || !X || !Yt || !B_values) return SPTIR_ERR_INVALID_ARG;
  const size_t b_bytes = sizeof(float) * (size_t)p->nnz;
  if (ranges_overlap(B_values, b_bytes, X, sizeof(float) * (size_t)p->n_rows * feat) ||
      ranges_overlap(B_values, b_bytes, Yt, sizeof(float) * (size_t)p->n_cols * feat))
    return SPTIR_ERR_INVALID_ARG;
  if (B_values != values && ranges_overlap(B_values, b_bytes, values, b_bytes)) return SPTIR_ERR_INVALID_ARG;
  hipStream_t stream = (hipStream_t)stream_;
  SddmmArgs a;
  a.indptr = p->indptr; a.indices = p->indices; a.values = values;
  a.X = X; a.Yt = Yt; a.B = B_values; a.nnz = p->nnz; a.n_rows = p->n_rows; a.feat = feat;
  a.e_row = p->e_row; a.e_col = p->e_col; a.e_pos = p->e_pos;
  a.run_first_entry = p->run_first_entry; a.run_len = p->run_len; a.xcd_run_ptr = p->xcd_run_ptr;
  const bool vec = vector_path_ok(X, Yt, feat);
  if (p->c == 1) {
    const int64_t runs = (p->nnz + kSddmmRun - 1) / kSddmmRun;
    dim3 grid((unsigned)((runs + kSddmmWaves - 1) / kSddmmWaves));
    if (!vec) hipLaunchKernelGGL(k_sddmm_generic<false>, grid, dim3(64 * kSddmmWaves), 0, stream, a);
    else launch_sddmm_for_feat<false>(a, grid, stream);
  } else {
    dim3 grid((unsigned)(8 * ((p->max_runs_per_xcd + kSddmmWaves - 1) / kSddmmWaves)));
    if (!vec) hipLaunchKernelGGL(k_sddmm_generic<true>, grid, dim3(64 * kSddmmWaves), 0, stream, a);
    else launch_sddmm_for_feat<true>(a, grid, stream);
  }
  SPTIR_HIP(hipGetLastError());
  return SPTIR_OK;
}

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
  a.e_row = a.e_col = a.e_pos = nullptr; a.run_first_entry = nullptr; a.run_len = nullptr; a.xcd_run_ptr = nullptr;
  if (!vector_path_ok(X, Yt, feat))
    hipLaunchKernelGGL(k_sddmm_generic<false>, grid, dim3(64 * kSddmmWaves), 0, stream, a);
  else launch_sddmm_for_feat<false>(a, grid, stream);
  SPTIR_HIP(hipGetLastError());
  return SPTIR_OK;
}
