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

#include <algorithm>
#include <mutex>
#include <new>
#include <vector>

#include "sptir_internal.h"
#include "sptir_scan.h"

namespace sptir {
namespace {

constexpr int kMaxBins = 32;  // k <= 30 -> bins 0..k plus the remainder bin k+1

struct BuildShape {
  int32_t n_rows, n_cols, c, k, w;
  int32_t nb;  // bins per partition = k + 2
  int32_t NB;  // row blocks = ceil(n_rows / 256)
};

// bound[(p - 1) * n_rows + r] = first position of row r whose column is >= p * w, for p = 1 .. c-1.  A workgroup
// takes kBoundRows rows x up to kBoundParts partitions with the partition index running fastest over the lanes, so
// that the searches of a wavefront probe the entries of a few rows only (they are in cache after the first
// probes), and writes its results through an LDS tile, so that consecutive lanes write consecutive rows.
constexpr int kBoundRows = 64, kBoundParts = 64;

__global__ __launch_bounds__(256) void k_piece_bounds(BuildShape s, int32_t nnz,
                                                      const int32_t* __restrict__ indptr,
                                                      const int32_t* __restrict__ indices,
                                                      int32_t* __restrict__ bound) {
  __shared__ int32_t tile[kBoundParts][kBoundRows + 1];
  const int n_pc = (s.c - 1 + kBoundParts - 1) / kBoundParts;
  const int rb = blockIdx.x / n_pc, pc = blockIdx.x % n_pc;
  const int r0 = rb * kBoundRows, p0 = 1 + pc * kBoundParts;
  const int np = s.c - p0 < kBoundParts ? s.c - p0 : kBoundParts;
  const int nr = s.n_rows - r0 < kBoundRows ? s.n_rows - r0 : kBoundRows;
  for (int idx = threadIdx.x; idx < nr * np; idx += blockDim.x) {
    const int rl = idx / np, pl = idx - rl * np;
    // (this runs before the host has seen the verdict on indptr: whatever it holds, no read leaves `indices`)
    int a = indptr[r0 + rl], b = indptr[r0 + rl + 1];
    a = a < 0 ? 0 : (a > nnz ? nnz : a);
    b = b < a ? a : (b > nnz ? nnz : b);
    tile[pl][rl] = lower_bound_col(indices, a, b, (int64_t)(p0 + pl) * s.w);
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < nr * np; idx += blockDim.x) {
    const int pl = idx / nr, rl = idx - pl * nr;
    bound[(int64_t)(p0 + pl - 1) * s.n_rows + r0 + rl] = tile[pl][rl];
  }
}

// start and length of row r's piece in partition p
__device__ __forceinline__ void row_piece(const BuildShape& s, const int32_t* __restrict__ indptr,
                                          const int32_t* __restrict__ bound, int r, int p, int* lo, int* len) {
  const int first = (p == 0) ? indptr[r] : bound[(int64_t)(p - 1) * s.n_rows + r];
  const int last = (p == s.c - 1) ? indptr[r + 1] : bound[(int64_t)p * s.n_rows + r];
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
// flags[4]: number of positions q >= 1 whose value differs (as a bit pattern) from the one stored before it
// flags[5]: number of non-empty rows whose first value differs from the value stored just before it
// Every row has one value for all of its entries iff flags[4] == flags[5] (only counted when `values` is given).
// The counters exist kFlagSlots times, 64 bytes apart, and a wavefront adds to the copy its workgroup id picks:
// tens of thousands of atomic adds to one address would take longer than reading the matrix.  The host adds up.
constexpr int kFlagSlots = 64, kFlagStride = 8;
__device__ __forceinline__ unsigned long long* flag_slot(unsigned long long* flags) {
  return flags + (blockIdx.x & (kFlagSlots - 1)) * kFlagStride;
}
__global__ void k_validate_rows(int32_t n_rows, int64_t nnz, const int32_t* __restrict__ indptr,
                                const int32_t* __restrict__ indices, const int32_t* __restrict__ values,
                                unsigned long long* flags) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  unsigned int legal_descents = 0, legal_changes = 0;
  bool bad = false;
  for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < n_rows; r += stride) {
    int64_t a = indptr[r], b = indptr[r + 1];
    const bool bad_here = (a < 0) || (b > nnz) || (a > b) || (r == 0 && a != 0) || (r == n_rows - 1 && b != nnz);
    bad |= bad_here;
    legal_descents += !bad_here && a < b && a > 0 && indices[a] <= indices[a - 1];
    if (values) legal_changes += !bad_here && a < b && a > 0 && values[a] != values[a - 1];
  }
  // a grid-wide count through one address: one atomic per wavefront, a few thousand in all
  for (int d = 32; d > 0; d >>= 1) {
    legal_descents += __shfl_down(legal_descents, d, 64);
    legal_changes += __shfl_down(legal_changes, d, 64);
  }
  const unsigned long long any_bad = __ballot(bad);
  flags = flag_slot(flags);
  if ((threadIdx.x & 63) == 0) {
    if (legal_changes) atomicAdd(&flags[5], (unsigned long long)legal_changes);
    if (legal_descents) atomicAdd(&flags[3], (unsigned long long)legal_descents);
    if (any_bad) flags[0] = 1;
  }
}

// One thread checks 8 consecutive positions per step (two 16-byte loads per array when `vec` says that the arrays
// are 16-byte aligned, 4-byte loads otherwise; all loads of a step are issued before any is used); position q is
// compared with position q - 1, which the lane below holds (the first lane of a wavefront loads it).
__device__ __forceinline__ int4 load4(const int32_t* __restrict__ p, int vec) {
  if (vec) return *reinterpret_cast<const int4*>(p);
  return make_int4(p[0], p[1], p[2], p[3]);
}
__device__ __forceinline__ int ascents_not(int prev, const int4& a, const int4& b, bool has_prev) {
  return (has_prev && a.x <= prev) + (a.y <= a.x) + (a.z <= a.y) + (a.w <= a.z) + (b.x <= a.w) + (b.y <= b.x) +
         (b.z <= b.y) + (b.w <= b.z);
}
__device__ __forceinline__ int changes_of(int prev, const int4& a, const int4& b, bool has_prev) {
  return (has_prev && a.x != prev) + (a.y != a.x) + (a.z != a.y) + (a.w != a.z) + (b.x != a.w) + (b.y != b.x) +
         (b.z != b.y) + (b.w != b.z);
}

__global__ __launch_bounds__(256) void k_validate_elems(int64_t nnz, int32_t n_cols, int vec,
                                                        const int32_t* __restrict__ indices,
                                                        const int32_t* __restrict__ values,
                                                        unsigned long long* flags) {
  constexpr int kPer = 8;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x * kPer;
  const int lane = threadIdx.x & 63;
  const bool with_values = values != nullptr;
  unsigned int descents = 0, changes = 0;
  bool range = false;
  int64_t q = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * kPer;
  for (; q + kPer <= nnz; q += stride) {  // whole groups
    const int64_t q_prev = q > 0 ? q - 1 : 0;
    const int4 c0 = load4(indices + q, vec), c1 = load4(indices + q + 4, vec);
    int4 v0 = make_int4(0, 0, 0, 0), v1 = v0;
    if (with_values) { v0 = load4(values + q, vec); v1 = load4(values + q + 4, vec); }
    int first_c = 0, first_v = 0;
    if (lane == 0) {
      first_c = indices[q_prev];
      if (with_values) first_v = values[q_prev];
    }
    int prev_c = __shfl_up(c1.w, 1, 64), prev_v = __shfl_up(v1.w, 1, 64);
    if (lane == 0) { prev_c = first_c; prev_v = first_v; }
    const unsigned n = (unsigned)n_cols;
    range |= ((unsigned)c0.x >= n) | ((unsigned)c0.y >= n) | ((unsigned)c0.z >= n) | ((unsigned)c0.w >= n) |
             ((unsigned)c1.x >= n) | ((unsigned)c1.y >= n) | ((unsigned)c1.z >= n) | ((unsigned)c1.w >= n);
    descents += ascents_not(prev_c, c0, c1, q > 0);
    if (with_values) changes += changes_of(prev_v, v0, v1, q > 0);
  }
  for (int i = 0; i < kPer && q + i < nnz; ++i) {  // the thread that holds the last, partial group
    const int32_t col = indices[q + i];
    range |= (unsigned)col >= (unsigned)n_cols;
    descents += (q + i > 0) && col <= indices[q + i > 0 ? q + i - 1 : 0];
    if (with_values) changes += (q + i > 0) && values[q + i] != values[q + i > 0 ? q + i - 1 : 0];
  }
  // a grid-wide count through one address: one atomic per wavefront, a few thousand in all
  for (int d = 32; d > 0; d >>= 1) {
    descents += __shfl_down(descents, d, 64);
    changes += __shfl_down(changes, d, 64);
  }
  unsigned long long any_range = __ballot(range);
  flags = flag_slot(flags);
  if ((threadIdx.x & 63) == 0) {
    if (changes) atomicAdd(&flags[4], (unsigned long long)changes);
    if (descents) atomicAdd(&flags[2], (unsigned long long)descents);
    if (any_range) flags[1] = 1;
  }
}

// row_val[r] = the value of row r's first entry (0 for an empty row)
__global__ void k_row_values(int32_t n_rows, const int32_t* __restrict__ indptr, const float* __restrict__ values,
                             float* row_val) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r < n_rows) row_val[r] = indptr[r + 1] > indptr[r] ? values[indptr[r]] : 0.f;
}

// --------------------------------------------------------------------- count
// counts   [c][nb][NB] int32 : pieces of each bin per row block
// rem_nnz  [c][NB]     int64 : non-zeros sent to the remainder per row block
__global__ __launch_bounds__(kBuildBlock) void k_count(BuildShape s, const int32_t* __restrict__ indptr,
                                                       const int32_t* __restrict__ bound, int32_t* counts,
                                                       int64_t* rem_nnz) {
  __shared__ int hist[kMaxBins];
  __shared__ unsigned long long sum_nnz;
  int tid = threadIdx.x;
  int p = blockIdx.x / s.NB, rb = blockIdx.x % s.NB;
  if (tid < kMaxBins) hist[tid] = 0;
  if (tid == 0) sum_nnz = 0;
  __syncthreads();
  int r = rb * kBuildBlock + tid;
  if (r < s.n_rows) {
    int lo, l;
    row_piece(s, indptr, bound, r, p, &lo, &l);
    if (l > 0) {
      int bin = bin_of_length(l, s.k);
      atomicAdd(&hist[bin], 1);
      if (bin == s.k + 1) atomicAdd(&sum_nnz, (unsigned long long)l);
    }
  }
  __syncthreads();
  if (tid < s.nb) counts[((int64_t)p * s.nb + tid) * s.NB + rb] = hist[tid];
  if (tid == 0) rem_nnz[(int64_t)p * s.NB + rb] = (int64_t)sum_nnz;
}

// ------------------------------------------------------------------- scatter
struct ScatterArgs {
  const int32_t* indptr;
  const int32_t* indices;
  const float* values;
  const int32_t* bound;        // piece boundaries (k_piece_bounds)
  const int32_t* counts;       // scanned: rank of the block's first piece of each bin
  const int64_t* rem_nnz;      // scanned
  const int64_t* bucket_row_ptr;
  const int64_t* bucket_slot_ptr;
  const int32_t* rem_part_ptr;
  const int64_t* rem_nnz_base;   // [c] first remainder nnz of each partition
  int32_t* row_ids;
  int32_t* cols;
  float* vals;
  int64_t* rem_ptr;
  int32_t* row_len;  // [R+M] real (unpadded) length of every ELL row and remainder piece
  int32_t* piece_of; // [c][n_rows] position in row_ids of the piece of (row, partition), -1 where the piece is empty
  int64_t R, S, M, T;
};

__global__ __launch_bounds__(kBuildBlock) void k_scatter(BuildShape s, ScatterArgs a) {
  __shared__ int wave_cnt[kWaves][kMaxBins];
  __shared__ long long wave_sums[kWaves];
  // the pieces of a wavefront, for the copy: slots before each piece, where it lies in the input, its real
  // length, where it goes
  __shared__ long long pre[kWaves][65];
  __shared__ unsigned pre32[kWaves][65];
  __shared__ long long piece_dst[kWaves][64];
  __shared__ int piece_lo[kWaves][64], piece_len[kWaves][64];
  int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // The c workgroups that copy the pieces of one block of rows read the same cache lines of the input (a piece
  // ends in the middle of a line, the next partition's starts there), so they are made neighbours in time and
  // share an XCD: workgroup ids go round the 8 XCDs, hence ids b, b + 8, b + 16, .. take consecutive work numbers.
  const long long n_work = (long long)gridDim.x, per_xcd = (n_work + 7) / 8;
  long long work = (long long)(blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  // (when the grid is not a multiple of 8 the last XCDs have one workgroup less: the numbers past the end wrap
  //  into the gaps those leave)
  const int full = (int)(n_work & 7);  // XCDs that have per_xcd workgroups (0: all of them)
  if (full != 0 && (int)(blockIdx.x & 7) >= full) work -= (int)(blockIdx.x & 7) - full;
  int rb = (int)(work / s.c), p = (int)(work % s.c);
  if (tid < kWaves * kMaxBins) (&wave_cnt[0][0])[tid] = 0;
  if (blockIdx.x == 0 && tid == 0) a.rem_ptr[a.M] = a.T;
  if (blockIdx.x == 0 && tid < kChunkSlots) {  // the spare entries past the end of the arrays
    a.row_ids[a.R + a.M + tid] = 0;
    a.cols[a.S + a.T + tid] = 0;
    a.vals[a.S + a.T + tid] = 0.f;
  }
  __syncthreads();

  int r = rb * kBuildBlock + tid;
  int lo = 0, l = 0, bin = -1;
  if (r < s.n_rows) {
    row_piece(s, a.indptr, a.bound, r, p, &lo, &l);
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

  // remainder pieces also need the running sum of their lengths
  bool is_rem = (bin == s.k + 1);
  long long my_nnz = is_rem ? l : 0;
  long long tot;
  long long nnz_before = block_exclusive_scan<long long>(my_nnz, wave_sums, &tot);
  // (block_exclusive_scan synchronises the workgroup, so wave_cnt is complete here)
  // Lanes without a piece stay alive with width 0: the wide copies below need all 64 lanes.
  int width = 0;
  int64_t dst = 0;
  int32_t where = -1;  // position of this piece in row_ids
  if (bin >= 0) {
    int before = 0;
    for (int wv = 0; wv < wave; ++wv) before += wave_cnt[wv][bin];
    int64_t q = (int64_t)a.counts[((int64_t)p * s.nb + bin) * s.NB + rb] + before + rank_in_wave;
    if (!is_rem) {
      int64_t b = (int64_t)p * (s.k + 1) + bin;
      width = 1 << bin;
      where = (int32_t)(a.bucket_row_ptr[b] + q);
      a.row_ids[where] = r;
      a.row_len[where] = l;
      dst = a.bucket_slot_ptr[b] + q * width;
    } else {
      int64_t m = (int64_t)a.rem_part_ptr[p] + q;
      int64_t t0 = a.rem_nnz_base[p] + a.rem_nnz[(int64_t)p * s.NB + rb] + nnz_before;
      where = (int32_t)(a.R + m);
      a.row_ids[where] = r;
      a.row_len[where] = l;
      a.rem_ptr[m] = t0;
      width = l;
      dst = a.S + t0;
    }
  }
  if (a.piece_of && r < s.n_rows) a.piece_of[(int64_t)p * s.n_rows + r] = where;
  // ---- the copy.  The pieces of a wavefront, `width` slots each (real entries, then pads: a pad repeats the last
  // real column and holds +0.0f), form one sequence; every step the 64 lanes take 64 consecutive slots of it, so
  // that lanes are busy whatever the lengths of the pieces and neighbouring lanes touch neighbouring addresses.
  long long inc = width;
  for (int d = 1; d < 64; d <<= 1) {
    const long long t = __shfl_up(inc, d, 64);
    if (lane >= d) inc += t;
  }
  if (lane == 0) { pre[wave][0] = 0; pre32[wave][0] = 0; }
  pre[wave][lane + 1] = inc;
  pre32[wave][lane + 1] = (unsigned)inc;
  piece_lo[wave][lane] = lo; piece_len[wave][lane] = l; piece_dst[wave][lane] = dst;
  __syncthreads();
  const long long total = pre[wave][64];
  const int32_t* __restrict__ indices = a.indices;
  const float* __restrict__ values = a.values;
  int32_t* __restrict__ cols = a.cols;
  float* __restrict__ vals = a.vals;
  if (total >= 0x7FFFFFFFll) {
    // (a wavefront with 2^31 slots or more: piece after piece, the 32-bit positions below do not reach)
    for (int i = 0; i < 64; ++i) {
      const long long width_i = pre[wave][i + 1] - pre[wave][i];
      const int len_i = piece_len[wave][i];
      for (long long j = lane; j < width_i; j += 64) {
        const long long src = piece_lo[wave][i] + (j < len_i ? j : (long long)len_i - 1);
        cols[piece_dst[wave][i] + j] = indices[src];
        vals[piece_dst[wave][i] + j] = j < len_i ? values[src] : 0.0f;
      }
    }
    return;
  }
  constexpr int kUnroll = 4;
  const unsigned total32 = (unsigned)total;
  for (unsigned f0 = 0; f0 < total32; f0 += 64 * kUnroll) {
    int32_t col[kUnroll];
    float val[kUnroll];
    long long at[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const unsigned f = f0 + u * 64 + lane;
      at[u] = -1; col[u] = 0; val[u] = 0.f;
      if (f < total32) {
        int i = 0;  // the piece with pre[i] <= f < pre[i + 1]
#pragma unroll
        for (int step = 32; step > 0; step >>= 1)
          if (pre32[wave][i + step] <= f) i += step;
        const int j = (int)(f - pre32[wave][i]);
        const int len_i = piece_len[wave][i];
        const bool real = j < len_i;
        const long long src = (long long)piece_lo[wave][i] + (real ? j : len_i - 1);
        col[u] = indices[src];
        val[u] = real ? values[src] : 0.0f;
        at[u] = piece_dst[wave][i] + j;
      }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
      if (at[u] >= 0) { cols[at[u]] = col[u]; vals[at[u]] = val[u]; }
  }
}

// ------------------------------------------------------- SpMM work-item list
// The SpMM kernel keeps the Y rows of one row block (row_block consecutive
// rows) in LDS and walks the real entries of the block's row pieces in chunks
// of kChunkSlots; a chunk never crosses a row-block boundary.  Rows ascend
// inside every bucket and inside every partition's remainder, hence the rows
// of a bin that fall into row block j are one contiguous run of row_ids; a
// "cell" holds the chunks that one (phase, row block, partition) contributes
// from one bin, or from its queues.  The cells of a (phase, row block) group
// are numbered partition by partition (see cells_per_group below) and their
// chunks are laid out in that order, so the chunks of a group are contiguous
// and sweep the column partitions in ascending order.
struct CellShape {
  int32_t c, k, nb;
  int32_t log2_rb, n_rb, ppg, n_phases;
  int32_t long_len;  // pieces with more real entries are not in the lists (heavy pieces)
  int64_t R;
};

// bin_rb_ptr[(p*nb + bin)*(n_rb+1) + j] = first position in row_ids of bin
// (p, bin) whose row id is >= j * row_block (absolute index into row_ids)
__global__ void k_cell_bounds(CellShape cs, const int64_t* __restrict__ bucket_row_ptr,
                              const int32_t* __restrict__ rem_part_ptr, const int32_t* __restrict__ row_ids,
                              int32_t* bin_rb_ptr) {
  int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t per_bin = (int64_t)cs.n_rb + 1;
  if (t >= (int64_t)cs.c * cs.nb * per_bin) return;
  int j = (int)(t % per_bin);
  int pb = (int)(t / per_bin);
  int p = pb / cs.nb, bin = pb % cs.nb;
  int64_t lo, hi;
  if (bin <= cs.k) {
    int64_t b = (int64_t)p * (cs.k + 1) + bin;
    lo = bucket_row_ptr[b]; hi = bucket_row_ptr[b + 1];
  } else {
    lo = cs.R + rem_part_ptr[p]; hi = cs.R + rem_part_ptr[p + 1];
  }
  int64_t bound = (int64_t)j << cs.log2_rb;
  while (lo < hi) {
    int64_t mid = lo + ((hi - lo) >> 1);
    if ((int64_t)row_ids[mid] < bound) lo = mid + 1; else hi = mid;
  }
  bin_rb_ptr[t] = (int32_t)lo;
}

// Cells of one (phase, row block) group, in chunk order: for every partition of the phase its nb bin cells
// (the chunks of that bin's rows that are cut wide) and one queue cell, then one pad cell that rounds the
// group's chunk count up to a multiple of kChunksPerQuad (the SpMM kernel fetches chunks four at a time).
//
// How the row pieces of a (group, partition) become chunks (pieces of at most long_len entries; bucket
// rows and remainder pieces alike, each with its real entries only):
//  * a piece is dealt whole to one of eight queues, one per lane group of the SpMM kernel, where its entries
//    follow those of the piece before it without a gap; chunk t of the queue cell holds entries 8t .. 8t+7 of
//    every queue, and the last entry of a piece carries a flag.  A lane group then walks whole rows alone,
//    keeps the running sum in registers, hands it over at a flag and needs no cross-lane reduction; no pad of
//    a bucket row is ever walked.  A piece goes to the queue that is shortest so far (buckets are visited
//    widest first, so this is the longest-first rule up to a factor of two);
//  * unless the piece is longer than a chunk and than an even share of what is still to be dealt: such a
//    piece is cut "wide" instead, into chunks of 64 entries that all eight lane groups share, in its bin's cell.
// The rows of one partition are distinct, so two queues never hand over the same row of Y in one instruction.
__device__ __forceinline__ int cells_per_part(const CellShape& cs) { return cs.nb + 1; }
__device__ __forceinline__ int cells_per_group(const CellShape& cs) { return cs.ppg * (cs.nb + 1) + 1; }

struct PiecePlace {     // where the entries of a queued row piece go (len 0: the piece is not queued)
  uint32_t slot0;       // its first slot in the fused (cols, vals) arrays (fewer than 2^32: at most 2 * nnz)
  int32_t first_chunk;  // first chunk of the queue cell
  int32_t where;        // position of its first entry in the queue | queue << 28
  int32_t len;          // real entries
};
static_assert(sizeof(PiecePlace) == 16, "PiecePlace must stay 16 bytes");
constexpr uint32_t kChunkIsQueue = 1u << 14;

__device__ __forceinline__ int chunks_of_length(int len) { return (len + kChunkSlots - 1) / kChunkSlots; }
inline int64_t chunks_of_slots(int64_t slots) { return (slots + kChunkSlots - 1) / kChunkSlots; }

// Walks the row pieces of partition p in row block rb and tells the visitor what becomes of each:
//   (pieces of more than cs.long_len entries are not part of the lists: the heavy-piece launch sums them)
//   v.on_wide(bin, q, len)                 cut into 64-entry chunks
//   v.on_queued(bin, q, len, g, start)     entries start .. start + len - 1 of queue g
//   v.on_dealt(load, chunks)               at the end: entries per queue, chunks of the queue cell
// and returns the chunks of the queue cell.
template <typename Visitor>
__device__ __forceinline__ int deal_partition(const CellShape& cs, const int32_t* __restrict__ bin_rb_ptr,
                                              const int32_t* __restrict__ row_len, int p, int rb, Visitor& v) {
  const int64_t per_bin = (int64_t)cs.n_rb + 1;
  long long to_deal = 0;  // entries not dealt yet
  for (int bin = 0; bin < cs.nb; ++bin) {
    const int32_t* ptr = bin_rb_ptr + ((int64_t)p * cs.nb + bin) * per_bin + rb;
    for (int32_t q = ptr[0]; q < ptr[1]; ++q) {
      const int len = row_len[q];
      if (len <= cs.long_len) to_deal += len;
    }
  }
  int load[8];
#pragma unroll
  for (int g = 0; g < 8; ++g) load[g] = 0;
  for (int bin = cs.nb - 1; bin >= 0; --bin) {
    const int32_t* ptr = bin_rb_ptr + ((int64_t)p * cs.nb + bin) * per_bin + rb;
    for (int32_t q = ptr[0]; q < ptr[1]; ++q) {
      const int len = row_len[q];
      if (len > cs.long_len) continue;
      const long long share = (to_deal + 7) >> 3;
      to_deal -= len;
      if (len > kChunkSlots && len > share) { v.on_wide(bin, q, len); continue; }
      int best = 0, best_load = load[0];
#pragma unroll
      for (int g = 1; g < 8; ++g)
        if (load[g] < best_load) { best_load = load[g]; best = g; }
      v.on_queued(bin, q, len, best, best_load);
#pragma unroll
      for (int g = 0; g < 8; ++g) load[g] += (g == best) ? len : 0;
    }
  }
  int longest = 0;
#pragma unroll
  for (int g = 0; g < 8; ++g) longest = max(longest, load[g]);
  const int chunks = (longest + 7) >> 3;
  v.on_dealt(load, chunks);
  return chunks;
}

// One thread per (group, partition of its phase): chunk counts of that partition's cells.
struct CountVisitor {
  long long* cell;  // the partition's nb + 1 counts
  __device__ void on_wide(int bin, int32_t, int len) { cell[bin] += chunks_of_length(len); }
  __device__ void on_queued(int, int32_t, int, int, int) {}
  __device__ void on_dealt(const int (&)[8], int) {}
};

__global__ void k_part_chunk_counts(CellShape cs, int64_t n_parts, const int32_t* __restrict__ bin_rb_ptr,
                                    const int32_t* __restrict__ row_len, long long* cell_chunks) {
  int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n_parts) return;
  const int64_t grp = t / cs.ppg;
  const int p_local = (int)(t % cs.ppg);
  const int rb = (int)(grp % cs.n_rb), phase = (int)(grp / cs.n_rb);
  const int p = phase * cs.ppg + p_local;
  long long* cell = cell_chunks + grp * cells_per_group(cs) + (int64_t)p_local * cells_per_part(cs);
  for (int i = 0; i <= cs.nb; ++i) cell[i] = 0;
  if (p >= cs.c) return;  // a partition past the last one
  CountVisitor v{cell};
  cell[cs.nb] = deal_partition(cs, bin_rb_ptr, row_len, p, rb, v);
}

// One thread per (phase, row block) group: the pad cell gets what is missing to a multiple of kChunksPerQuad,
// the group's counts become their exclusive prefix inside the group, group_total[grp] their sum.
__global__ __launch_bounds__(256) void k_group_scan(CellShape cs, int64_t n_groups, long long* cell_chunks,
                                                    long long* group_total, unsigned long long* longest) {
  // one wavefront per group: an exclusive scan over the group's cells, 64 at a time
  const int64_t grp = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (grp >= n_groups) return;
  const int lane = threadIdx.x & 63;
  const int cpg = cells_per_group(cs);
  long long* c = cell_chunks + grp * cpg;
  long long carry = 0;
  for (int i0 = 0; i0 < cpg - 1; i0 += 64) {
    const int i = i0 + lane;
    const long long n = i < cpg - 1 ? c[i] : 0;
    const long long incl = wave_inclusive_scan(n, lane);
    if (i < cpg - 1) c[i] = carry + incl - n;
    carry += __shfl(incl, 63, 64);
  }
  if (lane == 0) {
    c[cpg - 1] = carry;
    const long long padded = carry + (kChunksPerQuad - carry % kChunksPerQuad) % kChunksPerQuad;
    group_total[grp] = padded;
    // the longest list (the sort of the launch order needs to know how many digits can differ)
    // (one of kFlagSlots counters, for the reason given there; the report takes their maximum)
    if (padded > 0) atomicMax(longest + (grp & (kFlagSlots - 1)) * kFlagStride, (unsigned long long)padded);
  }
}

constexpr int kGroupSeq = 1024;  // groups per sequence of the two-level scan over group totals

// ------------------------------------------------------------ chunk stream
// What the SpMM kernel actually reads: the chunks as fixed records, in list
// order, so that the address of every record follows from its list position
// alone (no dependent descriptor load inside the gather loop).  Four
// consecutive chunks form a quad, fetched with one 16-byte load per lane and
// array.  The 12-byte form (3 KB per quad):
//   quad[  0..255]  column ids, chunk i at 64*i  (slots past the last real one repeat a real column)
//   quad[256..511]  values                        (slots past the last real one hold +0.0f)
//   quad[512..767]  per slot: row relative to the first row of the row block in bits 0..15,
//                   the chunk's log2w in bits 16..21, the hand-over flag in bit 22 (the chunk's, or in a
//                   queue chunk the slot's: the last entry of a row piece), bit 23: the slot belongs to no
//                   row (past the end of a queue); slots of a wide chunk past its last entry hold -1
// The compact form (2 KB per quad; the kernel's time goes with the bytes it has
// to pull from beyond L2, and every feature tile re-reads the stream) folds the
// row word into the column word, see kCompactColBits:
//   quad[  0..255]  column - first column of the launch | row << 20 | real << 27 | log2w code << 28 | hand-over << 31
//   quad[256..511]  values
struct StreamShape {
  int32_t* stream;
  int32_t unit;   // 1: no values array (every row of A has one value, kept aside)
  int32_t compact;
  int32_t log2_rb;
  int32_t phase_width;  // columns a launch covers
};

__device__ __forceinline__ void put_slot(const StreamShape& ss, int64_t chunk, int slot, int32_t col_word,
                                         int32_t val_bits, int32_t row_word) {
  constexpr int kQuadSlots = kChunkSlots * kChunksPerQuad;
  const int n_arrays = (ss.compact ? 2 : 3) - (ss.unit ? 1 : 0);  // [cols][vals unless unit][row words unless compact]
  int32_t* quad = ss.stream + (chunk / kChunksPerQuad) * (n_arrays * kQuadSlots);
  const int at = (int)(chunk % kChunksPerQuad) * kChunkSlots + slot;
  quad[at] = col_word;
  if (!ss.unit) quad[kQuadSlots + at] = val_bits;
  if (!ss.compact) quad[(n_arrays - 1) * kQuadSlots + at] = row_word;
}

// entry e of a queued piece
__device__ __forceinline__ void put_queue_entry(const StreamShape& ss, int64_t first_chunk, int where, int e,
                                                int32_t col, float val, int32_t row, bool last) {
  const int pos = (where & 0x0FFFFFFF) + e, g = (where >> 28) & 7;
  const int local_row = row & ((1 << ss.log2_rb) - 1);
  int32_t col_word, row_word = 0;
  if (ss.compact) {
    const uint32_t col_rel = (uint32_t)(col - (col / ss.phase_width) * ss.phase_width);
    col_word = (int32_t)(col_rel | ((uint32_t)local_row << kCompactColBits) | (1u << 27) | (3u << 28) |
                         ((uint32_t)last << 31));
  } else {
    col_word = col;
    row_word = local_row | (3 << 16) | ((int)last << 22);
  }
  put_slot(ss, first_chunk + (pos >> 3), g * 8 + (pos & 7), col_word, __float_as_int(val), row_word);
}

// One thread per (group, partition): writes the chunk descriptors the counts above announced, the place of
// every queued piece, and the slots past the end of each queue.
struct FillVisitor {
  const CellShape& cs;
  const StreamShape& ss;
  int p;
  int64_t first_chunk;          // of the partition's first cell
  const long long* cell;        // scanned counts: chunks of this group before each of the partition's cells ...
  long long cell0;              // ... minus those before its first cell
  const int32_t* row_ids;
  const int64_t* bucket_row_ptr;
  const int64_t* bucket_slot_ptr;
  const int64_t* rem_ptr;
  int64_t S;
  Chunk* chunks;
  PiecePlace* place;
  int wide_bin;                 // bin whose wide rows are being written, and the next free chunk of its cell
  int64_t wide_it;

  __device__ int64_t cell_first(int i) const { return first_chunk + (cell[i] - cell0); }
  __device__ int64_t slot_of(int bin, int32_t q) const {
    if (bin <= cs.k) {
      const int64_t b = (int64_t)p * (cs.k + 1) + bin;
      return bucket_slot_ptr[b] + (((int64_t)q - bucket_row_ptr[b]) << bin);
    }
    return S + rem_ptr[q - cs.R];
  }
  __device__ void on_wide(int bin, int32_t q, int len) {
    if (bin != wide_bin) { wide_bin = bin; wide_it = cell_first(bin); }
    const int64_t slot0 = slot_of(bin, q);
    for (int off = 0; off < len; off += kChunkSlots) {
      Chunk ck;
      ck.slot0 = slot0 + off; ck.row0 = q;
      const int count = len - off < kChunkSlots ? len - off : kChunkSlots;
      ck.meta = (uint32_t)kRowLog2W | ((uint32_t)count << 6) | (off + kChunkSlots >= len ? (1u << 13) : 0u);
      chunks[wide_it++] = ck;
    }
  }
  __device__ void on_queued(int bin, int32_t q, int len, int g, int start) {
    PiecePlace pl;
    pl.slot0 = (uint32_t)slot_of(bin, q); pl.first_chunk = (int32_t)cell_first(cs.nb);
    pl.where = start | (g << 28); pl.len = len;
    place[q] = pl;
  }
  __device__ void on_dealt(const int (&load)[8], int n_chunks) {
    const int64_t first = cell_first(cs.nb);
    for (int i = 0; i < n_chunks; ++i) {  // the slots of a queue chunk are written piece by piece, not from here
      Chunk ck;
      ck.slot0 = 0; ck.row0 = 0;
      ck.meta = 3u | ((uint32_t)kChunkSlots << 6) | kChunkIsQueue;
      chunks[first + i] = ck;
    }
#pragma unroll
    for (int g = 0; g < 8; ++g)  // past the end of a queue: zeros that belong to no row
      for (int pos = load[g]; pos < 8 * n_chunks; ++pos)
        put_slot(ss, first + (pos >> 3), g * 8 + (pos & 7), ss.compact ? (int32_t)(3u << 28) : 0, 0,
                 (3 << 16) | (1 << 23));
  }
};

__global__ void k_part_fill_chunks(CellShape cs, StreamShape ss, int64_t n_parts,
                                   const int32_t* __restrict__ bin_rb_ptr,
                                   const long long* __restrict__ cell_first_chunk,
                                   const long long* __restrict__ group_first_chunk,
                                   const long long* __restrict__ seq_first_chunk,
                                   const int32_t* __restrict__ row_len, const int32_t* __restrict__ row_ids,
                                   const int64_t* __restrict__ bucket_row_ptr,
                                   const int64_t* __restrict__ bucket_slot_ptr, const int64_t* __restrict__ rem_ptr,
                                   int64_t S, Chunk* chunks, PiecePlace* place, int64_t* rb_chunk_ptr,
                                   int64_t n_chunks_total) {
  int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n_parts) return;
  const int64_t grp = t / cs.ppg;
  const int p_local = (int)(t % cs.ppg);
  const int rb = (int)(grp % cs.n_rb), phase = (int)(grp / cs.n_rb);
  const int p = phase * cs.ppg + p_local;
  const long long* cell = cell_first_chunk + grp * cells_per_group(cs) + (int64_t)p_local * cells_per_part(cs);
  const int64_t group_first = group_first_chunk[grp] + seq_first_chunk[grp / kGroupSeq];
  if (p_local == 0) rb_chunk_ptr[(int64_t)phase * cs.n_rb + rb] = group_first;
  if (grp == 0 && p_local == 0) rb_chunk_ptr[(int64_t)cs.n_phases * cs.n_rb] = n_chunks_total;
  if (p >= cs.c) return;
  FillVisitor v{cs, ss, p, group_first + cell[0], cell, cell[0], row_ids, bucket_row_ptr, bucket_slot_ptr, rem_ptr, S,
                chunks, place, -1, 0};
  deal_partition(cs, bin_rb_ptr, row_len, p, rb, v);
}

// One lane per row piece, 64 pieces per wavefront: the entries of the wavefront's queued pieces form one
// sequence of which every step the lanes take 64 consecutive ones (as in k_scatter), each going to its place in
// its queue.
__global__ __launch_bounds__(256) void k_pack_pieces(int64_t n_pieces, StreamShape ss,
                                                     const PiecePlace* __restrict__ place,
                                                     const int32_t* __restrict__ row_ids,
                                                     const int32_t* __restrict__ cols,
                                                     const float* __restrict__ vals) {
  __shared__ int pre[4][65];
  __shared__ PiecePlace pl_of[4][64];
  __shared__ int32_t row_of[4][64];
  const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  PiecePlace pl;
  pl.slot0 = 0; pl.first_chunk = 0; pl.where = 0; pl.len = 0;
  int32_t row = 0;
  if (q < n_pieces) { pl = place[q]; row = row_ids[q]; }
  int inc = pl.len;
  for (int d = 1; d < 64; d <<= 1) {
    const int t = __shfl_up(inc, d, 64);
    if (lane >= d) inc += t;
  }
  if (lane == 0) pre[wave][0] = 0;
  pre[wave][lane + 1] = inc;
  pl_of[wave][lane] = pl;
  row_of[wave][lane] = row;
  __syncthreads();
  const int total = pre[wave][64];
  constexpr int kUnroll = 4;
  for (int f0 = 0; f0 < total; f0 += 64 * kUnroll) {
    int32_t col[kUnroll];
    float val[kUnroll];
    int piece[kUnroll], e[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int f = f0 + u * 64 + lane;
      piece[u] = -1; e[u] = 0; col[u] = 0; val[u] = 0.f;
      if (f < total) {
        int i = 0;  // the piece with pre[i] <= f < pre[i + 1]
#pragma unroll
        for (int step = 32; step > 0; step >>= 1)
          if (pre[wave][i + step] <= f) i += step;
        piece[u] = i;
        e[u] = f - pre[wave][i];
        const int64_t src = (int64_t)pl_of[wave][i].slot0 + e[u];
        col[u] = cols[src];
        val[u] = ss.unit ? 0.f : vals[src];
      }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
      if (piece[u] >= 0) {
        const PiecePlace& w = pl_of[wave][piece[u]];
        put_queue_entry(ss, w.first_chunk, w.where, e[u], col[u], val[u], row_of[wave][piece[u]], e[u] == w.len - 1);
      }
  }
}

// One wavefront per chunk of a wide row (and per padding chunk of a group); reads the canonical arrays
// through the descriptor.  Queue chunks are written by k_pack_pieces and k_part_fill_chunks.
__global__ __launch_bounds__(256) void k_pack_stream(int64_t n_chunks, StreamShape ss,
                                                     const Chunk* __restrict__ chunks,
                                                     const int32_t* __restrict__ row_ids,
                                                     const int32_t* __restrict__ cols,
                                                     const float* __restrict__ vals) {
  int64_t q = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (q >= n_chunks) return;
  int lane = threadIdx.x & 63;
  const Chunk ck = chunks[q];
  if (ck.meta & kChunkIsQueue) return;
  const int lw = (int)(ck.meta & 63u), count = (int)((ck.meta >> 6) & 127u);
  if (count == 0) {  // padding of a group: contributes nothing, hands nothing over
    put_slot(ss, q, lane, ss.compact ? (int32_t)0xF0000000u : 0, 0, -1);
    return;
  }
  const int hand_over = (int)((ck.meta >> 13) & 1u);
  const int o = lane < count ? lane : count - 1;
  const int64_t src = ck.slot0 + o;
  const int32_t rid = row_ids[ck.row0 + (o >> lw)];
  const bool real = lane < count;
  const int32_t col = cols[src];
  const float val = vals[src];
  const int local_row = rid & ((1 << ss.log2_rb) - 1);
  if (ss.compact) {
    const uint32_t col_rel = (uint32_t)(col - (col / ss.phase_width) * ss.phase_width);
    put_slot(ss, q, lane,
             (int32_t)(col_rel | ((uint32_t)local_row << kCompactColBits) | ((uint32_t)real << 27) |
                       ((uint32_t)(lw > 6 ? 7 : lw) << 28) | ((uint32_t)hand_over << 31)),
             real ? __float_as_int(val) : 0, 0);
  } else {
    put_slot(ss, q, lane, col, real ? __float_as_int(val) : 0,
             real ? (local_row | (lw << 16) | (hand_over << 22)) : -1);
  }
}

// ------------------------------------------------------------ heavy pieces
// A piece of more than heavy_len real entries is "heavy".  The entries of all heavy pieces form one sequence, in
// the order of row_ids (buckets in bucket order, then the remainder: partition-major), which is cut into 64-slot
// chunks.  When heavy_len >= kChunkSlots the pieces follow each other without a gap (a chunk then holds the end
// of at most one piece, which is what the kernel can hand over per chunk); shorter heavy pieces each start a
// chunk of their own.  Exclusive prefixes over the pieces:
//   unit_before[q]  heavy pieces before piece q
//   hent_before[q]  slots of the heavy sequence before piece q
// Both arrays have one element more than there are pieces, so that after the scan the last one is the total.
// *heavy_nnz receives the real entries of all heavy pieces.
__device__ __forceinline__ int heavy_footprint(int len, int heavy_len) {
  return heavy_len >= kChunkSlots ? len : chunks_of_length(len) * kChunkSlots;
}

__global__ void k_heavy_counts(int64_t n_pieces, const int32_t* __restrict__ row_len, int32_t heavy_len,
                               int32_t* unit_before, int32_t* hent_before, unsigned long long* heavy_nnz) {
  const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int len = q < n_pieces ? row_len[q] : 0;
  const bool heavy = len > heavy_len;
  if (q <= n_pieces) {
    unit_before[q] = heavy ? 1 : 0;
    hent_before[q] = heavy ? heavy_footprint(len, heavy_len) : 0;
  }
  unsigned long long mine = heavy ? (unsigned long long)len : 0ull;
  for (int d = 32; d > 0; d >>= 1) mine += __shfl_down(mine, d, 64);
  if ((threadIdx.x & 63) == 0 && mine) atomicAdd(flag_slot(heavy_nnz), mine);  // (kFlagSlots counters, see there)
}

constexpr int kScanSeq = 4096;  // elements per sequence of the device-wide scan

// What the host needs to know before it can size the stream, in one array: report[0] = chunks of all lists,
// [1] = entries of heavy pieces (the sum of the counters k_heavy_counts added to; the longest list is the maximum
// of the counters next to them), [2] = heavy pieces, [3] = slots of the heavy sequence, [4] = chunks of the longest
// list.
constexpr int kReport2 = 5;
__global__ void k_report(const long long* totals, const long long* heavy_nnz_slots, const int32_t* unit_before,
                         const int32_t* hent_before, int64_t n_pieces, long long* report) {
  const int i = threadIdx.x;
  if (i >= kReport2) return;
  long long v;
  if (i == 0) v = totals[0];
  else if (i == 1) { v = 0; for (int slot = 0; slot < kFlagSlots; ++slot) v += heavy_nnz_slots[slot * kFlagStride]; }
  else if (i == 2) v = unit_before ? unit_before[n_pieces] : 0;
  else if (i == 3) v = hent_before ? hent_before[n_pieces] : 0;
  else {
    v = 0;
    for (int slot = 0; slot < kFlagSlots; ++slot) {
      const long long o = heavy_nnz_slots[slot * kFlagStride + 1];
      v = o > v ? o : v;
    }
  }
  report[i] = v;
}

__global__ void k_pick2(const int32_t* a, const int32_t* b, int32_t* dst) {
  if (threadIdx.x == 0) { dst[0] = *a; dst[1] = *b; }
}

// data[i] += seq_base[i / kScanSeq]: the last step of the device-wide exclusive scan
__global__ void k_add_seq_base(int64_t n, int32_t* data, const int32_t* __restrict__ seq_base) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) data[i] += seq_base[i / kScanSeq];
}

// first slot of piece q in the fused (cols, vals) arrays
__device__ __forceinline__ int64_t piece_slot0(int64_t q, int64_t B, int32_t k, int64_t R, int64_t S,
                                               const int64_t* __restrict__ bucket_row_ptr,
                                               const int64_t* __restrict__ bucket_slot_ptr,
                                               const int64_t* __restrict__ rem_ptr) {
  if (q >= R) return S + rem_ptr[q - R];
  int64_t lo = 0, hi = B;  // last bucket b with bucket_row_ptr[b] <= q
  while (hi - lo > 1) {
    const int64_t mid = lo + ((hi - lo) >> 1);
    if (bucket_row_ptr[mid] <= q) lo = mid; else hi = mid;
  }
  const int bin = (int)(lo % (k + 1));
  return bucket_slot_ptr[lo] + ((q - bucket_row_ptr[lo]) << bin);
}

// One thread per piece: heavy piece number u notes where its slots start in the heavy sequence, where its real
// entries end there, and where its entries lie in the fused (cols, vals) arrays (unit_start, unit_end, unit_slot0;
// unit_start has one more element, the total).
__global__ void k_heavy_units(int64_t n_pieces, const int32_t* __restrict__ row_len,
                              const int32_t* __restrict__ unit_before, const int32_t* __restrict__ hent_before,
                              int64_t B, int32_t k, int64_t R, int64_t S,
                              const int64_t* __restrict__ bucket_row_ptr,
                              const int64_t* __restrict__ bucket_slot_ptr, const int64_t* __restrict__ rem_ptr,
                              int32_t heavy_len, int32_t* __restrict__ unit_start,
                              int32_t* __restrict__ unit_end, int64_t* __restrict__ unit_slot0,
                              int32_t* __restrict__ quad_unit) {
  const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (q > n_pieces) return;
  if (q == n_pieces) { unit_start[unit_before[q]] = hent_before[q]; return; }
  if (unit_before[q + 1] == unit_before[q]) return;
  const int u = unit_before[q];
  const int64_t start = hent_before[q], len = row_len[q];
  unit_start[u] = (int32_t)start;
  unit_end[u] = (int32_t)(start + len);
  unit_slot0[u] = piece_slot0(q, B, k, R, S, bucket_row_ptr, bucket_slot_ptr, rem_ptr);
  // every quad of the heavy sequence whose first slot lies in this piece learns so (the pieces follow each other
  // without a gap, so every quad that starts before the end of the sequence hears from exactly one piece)
  constexpr int kQuadSlots = kChunkSlots * kChunksPerQuad;
  const int64_t end = start + heavy_footprint((int)len, heavy_len);
  for (int64_t quad = (start + kQuadSlots - 1) / kQuadSlots; quad * kQuadSlots < end; ++quad) quad_unit[quad] = u;
}

// One wavefront per kPackRun consecutive chunks of the heavy sequence (a whole quad), a lane per slot: writes the
// chunks' stream records.  The slot words of a chunk all name the slot at which a piece ends in it (in the place of
// the local row of the list records), with the hand-over flag set if one does.  Which pieces a chunk covers is the
// same for all lanes: quad_unit names the piece the quad starts in, the walk over unit_start from there runs on
// wave-uniform values.
constexpr int kPackRun = kChunksPerQuad;

__global__ __launch_bounds__(256) void k_pack_heavy(int64_t n_heavy_chunks, int64_t first_chunk, StreamShape ss,
                                                    int32_t n_units, const int32_t* __restrict__ unit_start,
                                                    const int32_t* __restrict__ unit_end,
                                                    const int64_t* __restrict__ unit_slot0,
                                                    const int32_t* __restrict__ quad_unit,
                                                    const int32_t* __restrict__ cols, const float* __restrict__ vals) {
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int64_t ck0 = ((int64_t)blockIdx.x * (blockDim.x >> 6) + wave) * kPackRun;
  if (ck0 >= n_heavy_chunks) return;  // (n_heavy_chunks is a whole number of quads)
  const int lane = threadIdx.x & 63;
  const int64_t total = n_units > 0 ? (int64_t)unit_start[n_units] : 0;
  // the last unit that starts at or before the first slot of the run
  int lo = ck0 * kChunkSlots < total ? quad_unit[ck0 / kPackRun] : 0;
  int64_t src[kPackRun];
  int32_t word[kPackRun];  // everything of the record but the column
  bool pad[kPackRun];
#pragma unroll
  for (int i = 0; i < kPackRun; ++i) {
    const int64_t e0 = (ck0 + i) * kChunkSlots;
    pad[i] = e0 >= total;  // past the last piece: padding up to a whole quad
    src[i] = 0; word[i] = 0;
    if (pad[i]) continue;
    while (lo + 1 < n_units && (int64_t)unit_start[lo + 1] <= e0) ++lo;
    const int64_t start_lo = unit_start[lo], end_lo = unit_end[lo], slot0_lo = unit_slot0[lo];
    const bool has_next = lo + 1 < n_units;
    const int64_t start_hi = unit_start[lo + 1];  // (the total when lo is the last unit)
    const int64_t end_hi = has_next ? unit_end[lo + 1] : 0, slot0_hi = has_next ? unit_slot0[lo + 1] : 0;
    const int64_t e = e0 + lane;
    const bool second = has_next && e >= start_hi;
    const int64_t start = second ? start_hi : start_lo, len = (second ? end_hi : end_lo) - start;
    const int64_t j = e - start;
    const bool real = j < len;
    src[i] = (second ? slot0_hi : slot0_lo) + (real ? j : len - 1);
    // the piece that ends inside this chunk, if any, is the one the chunk starts in (a later one would have to
    // start and end here: heavy pieces are longer than that, or start a chunk of their own)
    const int64_t last = end_lo - 1 - e0;
    const int hand_over = last >= 0 && last < kChunkSlots;
    const int end_slot = hand_over ? (int)last : 0;
    if (ss.compact)
      word[i] = (int32_t)(((uint32_t)end_slot << kCompactColBits) | ((uint32_t)real << 27) | (7u << 28) |
                          ((uint32_t)hand_over << 31));
    else
      word[i] = real ? (end_slot | (kRowLog2W << 16) | (hand_over << 22)) : -1;
  }
  int32_t col[kPackRun];
  float val[kPackRun];
#pragma unroll
  for (int i = 0; i < kPackRun; ++i) {
    col[i] = cols[src[i]];
    val[i] = ss.unit ? 0.f : vals[src[i]];
  }
#pragma unroll
  for (int i = 0; i < kPackRun; ++i) {
    if (pad[i]) {
      put_slot(ss, first_chunk + ck0 + i, lane, ss.compact ? (int32_t)0xF0000000u : 0, 0, -1);
    } else if (ss.compact) {
      const bool real = (word[i] >> 27) & 1;
      put_slot(ss, first_chunk + ck0 + i, lane, (int32_t)((uint32_t)col[i] | (uint32_t)word[i]),
               real ? __float_as_int(val[i]) : 0, 0);
    } else {
      put_slot(ss, first_chunk + ck0 + i, lane, col[i], word[i] >= 0 ? __float_as_int(val[i]) : 0, word[i]);
    }
  }
}

// Heavy list w covers the chunks [w*L, (w+1)*L) of the heavy sequence.  A wavefront writes a partial-sum row at
// every piece end and one more where its list ends, so its first write goes to row (pieces that end before
// chunk w*L) + w.
__global__ void k_heavy_list_slots(int32_t n_lists, int32_t list_chunks, int32_t n_units,
                                   const int32_t* __restrict__ unit_end, int32_t* hlist_first_slot) {
  const int w = blockIdx.x * blockDim.x + threadIdx.x;
  if (w >= n_lists) return;
  const int64_t x = (int64_t)w * list_chunks * kChunkSlots;
  int lo = 0, hi = n_units;  // first unit whose real entries end beyond slot x
  while (lo < hi) {
    const int mid = lo + ((hi - lo) >> 1);
    if ((int64_t)unit_end[mid] <= x) lo = mid + 1; else hi = mid;
  }
  hlist_first_slot[w] = lo + w;
}

// The partial-sum rows of heavy piece number u whose real entries are the slots [e0, e1) of the heavy sequence:
// rows u + w for every heavy list w that holds one of them (see k_heavy_list_slots).
__device__ __forceinline__ void piece_slots(int list_chunks, int u, int e0, int e1, int* first, int* count) {
  const int per_list = list_chunks * kChunkSlots;
  const int w0 = e0 / per_list, w1 = (e1 - 1) / per_list;
  *first = u + w0;
  *count = w1 - w0 + 1;
}

// One thread per row: how many partial-sum rows the heavy pieces of the row have (row_slot_ptr before its scan)
__global__ void k_row_slot_counts(int32_t n_rows, int32_t c, int32_t list_chunks,
                                  const int32_t* __restrict__ piece_of,
                                  const int32_t* __restrict__ row_len, const int32_t* __restrict__ unit_before,
                                  const int32_t* __restrict__ hent_before, int32_t* row_slot_ptr) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r > n_rows) return;
  int n = 0;
  if (r < n_rows) {
    for (int p = 0; p < c; ++p) {
      const int32_t q = piece_of[(int64_t)p * n_rows + r];
      if (q < 0 || unit_before[q + 1] == unit_before[q]) continue;
      int first, count;
      piece_slots(list_chunks, unit_before[q], hent_before[q], hent_before[q] + row_len[q], &first, &count);
      n += count;
    }
  }
  row_slot_ptr[r] = n;
}

__global__ void k_row_slot_fill(int32_t n_rows, int32_t c, int32_t list_chunks,
                                const int32_t* __restrict__ piece_of,
                                const int32_t* __restrict__ row_len, const int32_t* __restrict__ unit_before,
                                const int32_t* __restrict__ hent_before, const int32_t* __restrict__ row_slot_ptr,
                                int32_t* row_slots) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= n_rows) return;
  int32_t* out = row_slots + row_slot_ptr[r];
  for (int p = 0; p < c; ++p) {
    const int32_t q = piece_of[(int64_t)p * n_rows + r];
    if (q < 0 || unit_before[q + 1] == unit_before[q]) continue;
    int first, count;
    piece_slots(list_chunks, unit_before[q], hent_before[q], hent_before[q] + row_len[q], &first, &count);
    for (int i = 0; i < count; ++i) *out++ = first + i;
  }
}

// heavy_rows (compacted): flags, then after their scan the rows themselves
__global__ void k_heavy_row_flags(int32_t n_rows, const int32_t* __restrict__ row_slot_ptr, int32_t* flag) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r > n_rows) return;
  flag[r] = (r < n_rows && row_slot_ptr[r + 1] > row_slot_ptr[r]) ? 1 : 0;
}
__global__ void k_heavy_row_fill(int32_t n_rows, const int32_t* __restrict__ row_slot_ptr,
                                 const int32_t* __restrict__ before, int32_t* heavy_rows) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= n_rows) return;
  if (row_slot_ptr[r + 1] > row_slot_ptr[r]) heavy_rows[before[r]] = r;
}

// --------------------------------------------------------------- host helpers
// Pinned host memory for the few small arrays a build exchanges with the device.  The blocks are kept for the life
// of the process (pinning memory costs more than a small build) and lent to one build at a time.
class PinnedPool {
 public:
  struct Buf { char* p = nullptr; size_t size = 0; };
  Buf acquire(size_t bytes) {
    {
      std::lock_guard<std::mutex> g(m_);
      for (size_t i = 0; i < free_.size(); ++i)
        if (free_[i].size >= bytes) {
          Buf b = free_[i];
          free_.erase(free_.begin() + (long)i);
          return b;
        }
    }
    Buf b;
    b.size = std::max<size_t>(bytes, 64 * 1024);
    void* p = nullptr;
    if (hipHostMalloc(&p, b.size, hipHostMallocPortable) != hipSuccess) { (void)hipGetLastError(); b.size = 0; return b; }
    b.p = (char*)p;
    return b;
  }
  void release(Buf b) {
    if (!b.p) return;
    {
      std::lock_guard<std::mutex> g(m_);
      if (free_.size() < 8) { free_.push_back(b); return; }
    }
    (void)hipHostFree(b.p);
  }

 private:
  std::mutex m_;
  std::vector<Buf> free_;
};
PinnedPool& pinned_pool() {
  static PinnedPool* pool = new PinnedPool();  // never destroyed: no HIP call at process exit
  return *pool;
}

struct Blob {  // bump allocator over one device allocation
  char* base = nullptr;
  size_t size = 0;
  size_t reserve(size_t bytes) {
    size_t off = size;
    size = (size + bytes + 255) & ~(size_t)255;
    return off;
  }
};

// Exclusive scan of data[0 .. n) in place on `stream`; data must have room for n rounded up to whole sequences
// (the tail is zeroed here), seq_base for one int per sequence plus one.
sptir_status_t device_exclusive_scan(int32_t* data, int64_t n, int32_t* seq_base, hipStream_t stream) {
  if (n <= 0) return SPTIR_OK;
  const int64_t n_seq = (n + kScanSeq - 1) / kScanSeq;
  if (n_seq * kScanSeq > n)
    SPTIR_HIP(hipMemsetAsync(data + n, 0, sizeof(int32_t) * (size_t)(n_seq * kScanSeq - n), stream));
  hipLaunchKernelGGL(k_scan_sequences<int32_t>, dim3((unsigned)n_seq), dim3(kBuildBlock), 0, stream, data,
                     (int32_t)kScanSeq, seq_base);
  hipLaunchKernelGGL(k_scan_sequences<int32_t>, dim3(1), dim3(kBuildBlock), 0, stream, seq_base, (int32_t)n_seq,
                     seq_base + n_seq);
  hipLaunchKernelGGL(k_add_seq_base, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, n, data, seq_base);
  SPTIR_HIP(hipGetLastError());
  return SPTIR_OK;
}
size_t scan_room(int64_t n) { return (size_t)((n + kScanSeq - 1) / kScanSeq) * kScanSeq; }

int log2_row_block_setting(int32_t n_rows, bool rounds, bool full_rows, const sptir_build_options_t& opt) {
  long v = opt.row_block;
  if ((v < 8 || v > 256 || (v & (v - 1))) && full_rows) {
    // 16 rows x 512 bytes: the same 8 KB of LDS per wavefront as 64 rows of a 128-byte tile
    v = 16;
    while (v > 8 && n_rows / v < 1024) v >>= 1;
  } else if (v < 8 || v > 256 || (v & (v - 1))) {
    // A wavefront walks the list of one row block alone and keeps the block's tile of Y in LDS:
    // 64 rows x 128 bytes = 8 KB next to its 4 KB (6 KB) chunk ring allow 12 wavefronts per CU.  Measured on
    // the two large graphs with a launch per partition: 32 rows cost 3 % (more lists, each rounded up to whole
    // chunks), 128 rows 12 - 25 % (fewer wavefronts per CU); the low-degree graphs do not care.  In rounds the
    // lists hold short pieces only and 128 rows win (fewer, longer lists: 6 % on the largest graph).  128 rows is
    // the most a compact record can address.
    v = rounds ? 128 : 64;
    // A launch has (row blocks x feature tiles) wavefronts.  With one or two tiles (feat <= 64) that is too few
    // to balance 3,000 wavefront slots, and smaller row blocks win (measured at feat = 32: 32 rows 21 % faster).
    const long tiles = opt.feat_hint > 0 ? (opt.feat_hint + 31) / 32 : 4;
    while (v > 16 && (n_rows / v) * tiles < 6144) v >>= 1;
    // ... but keep at least ~1024 row blocks, or the 256 CUs do not fill
    while (v > 8 && n_rows / v < 1024) v >>= 1;
  }
  int l = 0;
  while ((1L << l) < v) ++l;
  return l;
}

// Do the X rows of a column partition have to be kept L2-resident while they are gathered (section 4.2.1's reason
// for column partitions)?  Only when rows are long: the gathers of a low-degree graph come from beyond L2 either
// way (measured: 8 slots per row and 4 partitions run 1.7x faster without any ordering by partition).  `fit`
// receives the partitions whose 128-byte-wide slices fit 2.5 MB of an XCD's 4 MB L2 together.
bool partitions_matter(int32_t c, int32_t w, int32_t n_rows, int64_t slots, long* fit_out) {
  const double slice_bytes = (double)w * 128.0;               // one 32-float tile of a partition's X rows
  long fit = (long)(2.5 * 1024 * 1024 / (slice_bytes > 1 ? slice_bytes : 1));
  if (fit < 1) fit = 1;
  *fit_out = fit;
  if (fit >= c) return false;
  const long phases = (c + fit - 1) / fit;
  const double slots_per_row = n_rows > 0 ? (double)slots / n_rows : 0.0;
  return slots_per_row >= 16.0 * (double)(phases - 1);
}

// A wavefront walks a chunk list alone, so the longest list bounds a launch from below, and the lists of a round
// run only as fast as the longest of them.  A piece with more entries than two average lists (at least 256, at
// most kHeavyLenMax) therefore leaves the lists (measured on the 169,343-row graph with rows of up to 13,000
// entries: SpMM 0.134 -> 0.11 ms).  In rounds every piece longer than one chunk does: what stays in the lists is
// then so even that the wavefronts of a round sweep the column partitions nearly in step.
int32_t heavy_len_setting(int64_t nnz, int64_t n_lists, bool rounds, const sptir_build_options_t& opt) {
  if (opt.heavy_len >= 1) return opt.heavy_len;
  if (rounds) return kChunkSlots;
  // (the heavy-piece launches cost some 8 microseconds of their own: not worth it on a graph that is done in 10)
  if (nnz < (1 << 19)) return kHeavyLenMax;
  const int64_t per_list = n_lists > 0 ? nnz / n_lists : 0;
  return (int32_t)std::min<int64_t>(kHeavyLenMax, std::max<int64_t>(256, 2 * per_list));
}

}  // namespace

sptir_build_options_t complete_options(const sptir_build_options_t* given) {
  sptir_build_options_t o;
  memset(&o, 0, sizeof(o));
  if (given) {
    size_t n = given->struct_size > 0 ? (size_t)given->struct_size : 0;
    if (n > sizeof(o)) n = sizeof(o);
    memcpy(&o, given, n);
  }
  o.struct_size = (int32_t)sizeof(o);
  return o;
}

LaunchShape decide_launch_shape(int32_t n_rows, int32_t n_cols, int32_t c, int32_t w, int64_t stored_slots,
                                const sptir_build_options_t& opt) {
  LaunchShape ls;
  long fit = 1;
  const bool matter = partitions_matter(c, w, n_rows, stored_slots, &fit);
  // rounds: every list sweeps all partitions, Y stays on chip and is written once; otherwise a launch per group
  // of partitions that reads back what the one before it wrote
  const bool parts_given = opt.parts_per_launch >= 1 && opt.parts_per_launch <= c;
  // (rounds pay when the pieces that stay in the lists are short: a read-modify-write of Y per partition then
  //  costs as much as the pieces themselves; with long pieces the wavefronts of a round, which nothing holds in
  //  step, lose more by drifting onto different partitions.  Measured: mean piece of 8 entries, 1.54 -> 1.04 ms;
  //  of 37 entries, 1.11 -> 1.39 ms.)
  const bool short_pieces = opt.light_piece_len == 0 || opt.light_piece_len < 16;
  ls.rounds = opt.rounds == 1 ? 1 : opt.rounds == 2 ? 0 : (matter && !parts_given && short_pieces ? 1 : 0);
  // Whole 512-byte runs of X per entry: only when asked for.  Measured at feat = 128 against the 128-byte tiles
  // bound to XCDs: 7 entries per row 0.108 -> 0.151 ms, 4.5 per row 0.037 -> 0.090 ms, 300 per row
  // 1.09 -> 1.66 ms.  Two lane groups instead of eight meet every queue four times per chunk, so partial sums go
  // through LDS at every step, and every XCD's L2 then sees all of X instead of a quarter of it.
  ls.full_rows = opt.full_rows == 1 ? 1 : 0;
  ls.log2_row_block = log2_row_block_setting(n_rows, ls.rounds != 0, ls.full_rows != 0, opt);
  if (ls.rounds) ls.parts_per_phase = c;
  else if (parts_given) ls.parts_per_phase = opt.parts_per_launch;
  else ls.parts_per_phase = matter ? (int32_t)fit : c;
  // a compact record holds a column in kCompactColBits bits and a row of the row block in 7
  const int64_t max_span = (int64_t)1 << kCompactColBits;
  ls.compact = (!opt.wide_stream && n_cols <= max_span && ls.log2_row_block <= kCompactMaxLog2RowBlock) ? 1 : 0;
  ls.n_phases = (c + ls.parts_per_phase - 1) / ls.parts_per_phase;
  return ls;
}

}  // namespace sptir

using namespace sptir;

extern "C" sptir_status_t sptir_hyb_build(const sptir_csr_t* csr, int32_t n_col_parts, int32_t max_bucket_log2,
                                          void* stream_, sptir_hyb_t** out) {
  return sptir::hyb_build_impl(csr, n_col_parts, max_bucket_log2, sptir::complete_options(nullptr), stream_, out);
}

extern "C" sptir_status_t sptir_hyb_build_ex(const sptir_csr_t* csr, int32_t n_col_parts, int32_t max_bucket_log2,
                                             const sptir_build_options_t* options, void* stream_, sptir_hyb_t** out) {
  const sptir_build_options_t opt = sptir::complete_options(options);
  if (opt.row_block != 0 && (opt.row_block < 8 || opt.row_block > 256 || (opt.row_block & (opt.row_block - 1))))
    return SPTIR_ERR_INVALID_ARG;
  if (opt.parts_per_launch < 0 || opt.rounds < 0 || opt.rounds > 2 || opt.heavy_len < 0 || opt.sweep_kb < 0 ||
      opt.feat_hint < 0 || opt.full_rows < 0 || opt.full_rows > 2)
    return SPTIR_ERR_INVALID_ARG;
  return sptir::hyb_build_impl(csr, n_col_parts, max_bucket_log2, opt, stream_, out);
}

sptir_status_t sptir::hyb_build_impl(const sptir_csr_t* csr, int32_t n_col_parts, int32_t max_bucket_log2,
                                     const sptir_build_options_t& opt, void* stream_, sptir_hyb_t** out) {
  const bool with_spmm_plan = !opt.no_spmm_plan;
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
  const int64_t n_pair_blocks = (int64_t)s.NB * s.c;
  if (n_pair_blocks > 0x7FFFFFFF) return SPTIR_ERR_OVERFLOW;
  const int64_t B = (int64_t)s.c * (s.k + 1);
  if (B > 0x7FFFFFFF) return SPTIR_ERR_OVERFLOW;

  sptir_alloc_fn alloc; sptir_free_fn free_; void* actx;
  current_allocator(&alloc, &free_, &actx);

  // ---- temporary storage: one device blob now, a second one once the cell count is known; one pinned host block
  // for everything that crosses to or from the host (pageable memory would make every small copy a blocking one)
  const size_t nbk = (size_t)(s.NB ? s.NB : 1);
  Blob tmp;
  // (flags, tot_rnnz and tot_bins lie next to each other: one copy brings them to the host)
  const size_t o_flags = tmp.size;
  tmp.size += kFlagSlots * kFlagStride * sizeof(unsigned long long);
  const size_t o_tot_rnnz = tmp.size;
  tmp.size += sizeof(int64_t) * (size_t)s.c;
  const size_t o_tot_bins = tmp.size;
  const size_t report1_bytes = tmp.reserve(sizeof(int32_t) * (size_t)s.c * s.nb) + sizeof(int32_t) * (size_t)s.c * s.nb;
  const size_t o_counts = tmp.reserve(sizeof(int32_t) * (size_t)s.c * s.nb * nbk);
  const size_t o_rnnz = tmp.reserve(sizeof(int64_t) * (size_t)s.c * nbk);
  const size_t o_rnnz_base = tmp.reserve(sizeof(int64_t) * (size_t)s.c);
  const size_t o_bound = tmp.reserve(sizeof(int32_t) * (size_t)(s.c - 1) * (size_t)(s.n_rows ? s.n_rows : 1) + 16);
  const size_t o_totals = tmp.reserve(sizeof(long long) * 4);  // chunks of all lists; -; longest list
  const size_t o_nnz_slots = tmp.reserve(sizeof(long long) * kFlagSlots * kFlagStride);  // entries of heavy pieces
  const size_t report2_count = kReport2;
  const size_t o_report2 = tmp.reserve(sizeof(long long) * report2_count);
  const size_t o_report3 = tmp.reserve(sizeof(int32_t) * 2);
  const int64_t n_bound_blocks =
      (((int64_t)s.n_rows + kBoundRows - 1) / kBoundRows) * (((int64_t)s.c - 1 + kBoundParts - 1) / kBoundParts);
  if (n_bound_blocks > 0x7FFFFFFF) return SPTIR_ERR_OVERFLOW;
  Blob host;
  const size_t h_report1 = host.reserve(report1_bytes);
  const size_t h_row_ptr = host.reserve(sizeof(int64_t) * (size_t)(B + 1));
  const size_t h_slot_ptr = host.reserve(sizeof(int64_t) * (size_t)(B + 1));
  const size_t h_rem_part_ptr = host.reserve(sizeof(int32_t) * (size_t)(s.c + 1));
  const size_t h_rnnz_base = host.reserve(sizeof(int64_t) * (size_t)s.c);
  const size_t h_report2 = host.reserve(sizeof(long long) * report2_count);
  const size_t h_report3 = host.reserve(sizeof(int32_t) * 4);
  const size_t h_misc = host.reserve(64);
  PinnedPool::Buf pinned = pinned_pool().acquire(host.size);
  if (!pinned.p) return SPTIR_ERR_ALLOC;
  host.base = pinned.p;
  tmp.base = (char*)scratch_alloc(tmp.size, alloc, actx, stream);
  if (!tmp.base) { pinned_pool().release(pinned); return SPTIR_ERR_ALLOC; }
  Blob tmp2;
  void* tmp_chunks = nullptr;
  void* tmp_place = nullptr;
  void* tmp_order = nullptr;

  sptir_hyb* h = new (std::nothrow) sptir_hyb();
  if (!h) { scratch_free(tmp.base, free_, actx); pinned_pool().release(pinned); return SPTIR_ERR_ALLOC; }
  memset(h, 0, sizeof(*h));
  h->alloc = alloc; h->free_ = free_; h->alloc_ctx = actx;
  h->n_rows = s.n_rows; h->n_cols = s.n_cols; h->c = s.c; h->k = s.k; h->w = s.w;
  h->nnz = csr->nnz; h->B = B;

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
    int32_t* d_tot_bins = (int32_t*)(tmp.base + o_tot_bins);
    int64_t* d_tot_rnnz = (int64_t*)(tmp.base + o_tot_rnnz);
    int64_t* d_rnnz_base = (int64_t*)(tmp.base + o_rnnz_base);
    int32_t* d_bound = (int32_t*)(tmp.base + o_bound);
    long long* d_totals = (long long*)(tmp.base + o_totals);
    long long* d_nnz_slots = (long long*)(tmp.base + o_nnz_slots);
    long long* d_report2 = (long long*)(tmp.base + o_report2);
    int32_t* d_report3 = (int32_t*)(tmp.base + o_report3);

    // ---- validation of the CSR input, and with it (their results are only used if the input is valid, and they
    // read nothing at a position the input names without clamping it) the piece boundaries, histogram and scans
    const unsigned long long* flag_slots = (const unsigned long long*)(host.base + h_report1);
    unsigned long long flags[6] = {0, 0, 0, 0, 0, 0};
    const int64_t* tot_rnnz = (const int64_t*)(host.base + h_report1 + (o_tot_rnnz - o_flags));
    const int32_t* tot_bins = (const int32_t*)(host.base + h_report1 + (o_tot_bins - o_flags));
    // (values are only looked at when a value-less stream is an option)
    const int32_t* value_bits = (with_spmm_plan && !opt.keep_values) ? (const int32_t*)csr->values : nullptr;
    BUILD_HIP(hipMemsetAsync(d_flags, 0, report1_bytes, stream));
    if (s.n_rows > 0)
      hipLaunchKernelGGL(k_validate_rows, dim3((unsigned)std::min<int64_t>(((int64_t)s.n_rows + 255) / 256, 4096)),
                         dim3(256), 0, stream, s.n_rows, csr->nnz,
                         csr->indptr, csr->indices, value_bits, d_flags);
    if (csr->nnz > 0)
      hipLaunchKernelGGL(k_validate_elems, dim3((unsigned)std::min<int64_t>((csr->nnz + 2047) / 2048, 8192)),
                         dim3(256), 0, stream, csr->nnz, s.n_cols,
                         (int)((((uintptr_t)csr->indices | (uintptr_t)csr->values) & 15) == 0), csr->indices,
                         value_bits, d_flags);
    if (s.NB > 0) {
      if (n_bound_blocks > 0)
        hipLaunchKernelGGL(k_piece_bounds, dim3((unsigned)n_bound_blocks), dim3(256), 0, stream, s, (int32_t)csr->nnz,
                           csr->indptr, csr->indices, d_bound);
      hipLaunchKernelGGL(k_count, dim3((unsigned)n_pair_blocks), dim3(kBuildBlock), 0, stream, s, csr->indptr,
                         d_bound, d_counts, d_rnnz);
      hipLaunchKernelGGL(k_scan_sequences<int32_t>, dim3((unsigned)(s.c * s.nb)), dim3(kBuildBlock), 0, stream,
                         d_counts, s.NB, d_tot_bins);
      hipLaunchKernelGGL(k_scan_sequences<long long>, dim3((unsigned)s.c), dim3(kBuildBlock), 0, stream,
                         (long long*)d_rnnz, s.NB, (long long*)d_tot_rnnz);
    }
    BUILD_HIP(hipGetLastError());
    BUILD_HIP(hipMemcpyAsync(host.base + h_report1, d_flags, report1_bytes, hipMemcpyDeviceToHost, stream));
    BUILD_HIP(hipStreamSynchronize(stream));
    for (int slot = 0; slot < kFlagSlots; ++slot)
      for (int i = 0; i < 6; ++i) flags[i] += flag_slots[slot * kFlagStride + i];
    bool bad_indptr = flags[0] != 0;
    if (s.n_rows == 0) {
      int32_t* first = (int32_t*)(host.base + h_misc);
      BUILD_HIP(hipMemcpyAsync(first, csr->indptr, sizeof(int32_t), hipMemcpyDeviceToHost, stream));
      BUILD_HIP(hipStreamSynchronize(stream));
      if (*first != 0 || csr->nnz != 0) bad_indptr = true;
    }
    if (bad_indptr) { st = SPTIR_ERR_INVALID_ARG; goto fail; }
    if (flags[1] || flags[2] != flags[3]) { st = SPTIR_ERR_UNSORTED; goto fail; }

    // ---- sizes and the small prefix arrays (host)
    int64_t* row_ptr = (int64_t*)(host.base + h_row_ptr);
    int64_t* slot_ptr = (int64_t*)(host.base + h_slot_ptr);
    int32_t* rem_part_ptr = (int32_t*)(host.base + h_rem_part_ptr);
    int64_t* rnnz_base = (int64_t*)(host.base + h_rnnz_base);
    int64_t M = 0, T = 0;
    row_ptr[0] = 0; slot_ptr[0] = 0; rem_part_ptr[0] = 0;
    for (int32_t p = 0; p < s.c; ++p) {
      for (int32_t i = 0; i <= s.k; ++i) {
        int64_t b = (int64_t)p * (s.k + 1) + i;
        int64_t rows = tot_bins[(size_t)p * s.nb + i];
        row_ptr[b + 1] = row_ptr[b] + rows;
        slot_ptr[b + 1] = slot_ptr[b] + (rows << i);
      }
      rnnz_base[p] = T;
      M += tot_bins[(size_t)p * s.nb + s.k + 1];
      T += tot_rnnz[p];
      if (M > 0x7FFFFFFF) { st = SPTIR_ERR_OVERFLOW; goto fail; }
      rem_part_ptr[p + 1] = (int32_t)M;
    }
    h->R = row_ptr[B]; h->S = slot_ptr[B]; h->M = M; h->T = T;
    if (h->R + h->M > 0x7FFFFFFF || h->S + T >= 0xFFFFFFFFll) { st = SPTIR_ERR_OVERFLOW; goto fail; }

    // ---- launch shape of the SpMM: row blocks, lists, heavy pieces
    CellShape cs;
    cs.c = s.c; cs.k = s.k; cs.nb = s.nb; cs.R = h->R;
    // mean real length of the pieces of at most kChunkSlots entries, estimated from the bucket sizes
    // (bucket i holds lengths 2^(i-1)+1 .. 2^i)
    sptir_build_options_t opt_here = opt;
    if (opt_here.light_piece_len == 0) {
      double pieces = 0, entries = 0;
      for (int32_t p = 0; p < s.c; ++p)
        for (int32_t i = 0; i <= s.k && (1 << i) <= kChunkSlots; ++i) {
          const double n = tot_bins[(size_t)p * s.nb + i];
          pieces += n;
          entries += n * (i == 0 ? 1.0 : 0.5 * ((1 << (i - 1)) + 1 + (1 << i)));
        }
      opt_here.light_piece_len = pieces > 0 ? std::max(1, (int)(entries / pieces + 0.5)) : 0;
    }
    const LaunchShape ls = decide_launch_shape(s.n_rows, s.n_cols, s.c, s.w, h->S + h->T, opt_here);
    cs.ppg = ls.parts_per_phase; cs.log2_rb = ls.log2_row_block; cs.n_phases = ls.n_phases;
    h->compact_stream = ls.compact;
    h->rounds = ls.rounds;
    h->full_rows = ls.full_rows;
    // Every row has one value for all its entries (a row-normalised adjacency matrix, say): the stream
    // carries no values, the kernels sum rows of X and scale each row of Y once.
    const bool one_value_per_row = value_bits && csr->nnz > 0 && flags[4] == flags[5];
    h->sweep_kb = opt.sweep_kb;  // (0: the defaults of the two sweep rules)
    cs.n_rb = (int32_t)(((int64_t)s.n_rows + (1 << cs.log2_rb) - 1) >> cs.log2_rb);
    cs.long_len = heavy_len_setting(csr->nnz, (int64_t)cs.n_phases * cs.n_rb, ls.rounds != 0, opt);
    h->heavy_len = cs.long_len;
    if (!with_spmm_plan) cs.n_rb = 0;  // no row blocks, no cells, no chunks: only the canonical arrays are built
    h->spmm_plan = with_spmm_plan ? 1 : 0;
    h->log2_row_block = cs.log2_rb; h->n_row_blocks = cs.n_rb;
    h->parts_per_phase = cs.ppg; h->n_phases = cs.n_phases;
    const int64_t n_pieces = h->R + M;
    const int64_t n_groups = (int64_t)cs.n_phases * cs.n_rb;
    const int64_t n_cells = n_groups * ((int64_t)cs.ppg * (cs.nb + 1) + 1);
    const int64_t n_parts = n_groups * cs.ppg;
    const int64_t n_bounds = (int64_t)s.c * s.nb * ((int64_t)cs.n_rb + 1);
    if (n_cells > 0x7FFFFFFF || n_bounds > 0x7FFFFFFF) { st = SPTIR_ERR_OVERFLOW; goto fail; }
    const size_t o_bounds = tmp2.reserve(sizeof(int32_t) * (size_t)(n_bounds ? n_bounds : 1));
    const size_t o_cell_chunks = tmp2.reserve(sizeof(long long) * (size_t)(n_cells ? n_cells : 1));
    const int64_t n_seq = (n_groups + kGroupSeq - 1) / kGroupSeq;
    const size_t o_group_tot = tmp2.reserve(sizeof(long long) * (size_t)(n_seq ? n_seq * kGroupSeq : 1));
    const size_t o_seq_tot = tmp2.reserve(sizeof(long long) * (size_t)(n_seq ? n_seq : 1));
    // heavy pieces: the two prefix arrays over the pieces, the (row, partition) -> piece map, scan scratch
    const bool want_heavy = with_spmm_plan && n_pieces > 0;
    const size_t o_unit = tmp2.reserve(sizeof(int32_t) * (want_heavy ? scan_room(n_pieces + 1) : 1));
    const size_t o_hent = tmp2.reserve(sizeof(int32_t) * (want_heavy ? scan_room(n_pieces + 1) : 1));
    const size_t o_piece_of = tmp2.reserve(sizeof(int32_t) * (want_heavy ? (size_t)s.c * (size_t)s.n_rows : 1));
    const size_t o_seq_base = tmp2.reserve(sizeof(int32_t) * 2 * (scan_room(std::max<int64_t>(n_pieces + 1, s.n_rows + 1)) / kScanSeq + 2));
    const size_t o_row_flags = tmp2.reserve(sizeof(int32_t) * (want_heavy ? scan_room((int64_t)s.n_rows + 1) : 1));
    tmp2.base = (char*)scratch_alloc(tmp2.size, alloc, actx, stream);
    if (!tmp2.base) { st = SPTIR_ERR_ALLOC; goto fail; }
    int32_t* d_bounds = (int32_t*)(tmp2.base + o_bounds);
    long long* d_cell_chunks = (long long*)(tmp2.base + o_cell_chunks);
    long long* d_group_tot = (long long*)(tmp2.base + o_group_tot);
    long long* d_seq_tot = (long long*)(tmp2.base + o_seq_tot);
    int32_t* d_unit = (int32_t*)(tmp2.base + o_unit);
    int32_t* d_hent = (int32_t*)(tmp2.base + o_hent);
    int32_t* d_piece_of = want_heavy ? (int32_t*)(tmp2.base + o_piece_of) : nullptr;
    int32_t* d_seq_base = (int32_t*)(tmp2.base + o_seq_base);
    int32_t* d_row_flags = (int32_t*)(tmp2.base + o_row_flags);

    // ---- the handle's device arrays whose sizes are known now: two allocations (cols and vals can be released
    // on their own); the arrays of the SpMM plan follow further down
    {
      Blob ba, bb;
      const size_t a_row_ptr = ba.reserve(sizeof(int64_t) * (size_t)(B + 1));
      const size_t a_slot_ptr = ba.reserve(sizeof(int64_t) * (size_t)(B + 1));
      const size_t a_rem_part = ba.reserve(sizeof(int32_t) * (size_t)(s.c + 1));
      const size_t a_rem_ptr = ba.reserve(sizeof(int64_t) * (size_t)(M + 1));
      // (row_ids, cols and vals end in kChunkSlots spare zero entries: whole 64-slot chunks are read from them
      //  when the stream is packed, the last one of an array may be shorter)
      const size_t a_row_ids = ba.reserve(sizeof(int32_t) * (size_t)(h->R + M + kChunkSlots));
      const size_t a_row_len = ba.reserve(sizeof(int32_t) * (size_t)(h->R + M + 1));
      const size_t a_rb_chunk = ba.reserve(sizeof(int64_t) * ((size_t)cs.n_phases * cs.n_rb + 1));
      const size_t a_row_val = ba.reserve(one_value_per_row ? sizeof(float) * (size_t)s.n_rows : 0);
      const size_t a_row_slot = ba.reserve(want_heavy ? sizeof(int32_t) * scan_room((int64_t)s.n_rows + 1) : 0);
      const size_t b_cols = bb.reserve(sizeof(int32_t) * (size_t)(h->S + T + kChunkSlots));
      const size_t b_vals = bb.reserve(sizeof(float) * (size_t)(h->S + T + kChunkSlots));
      h->blobs[0] = alloc(ba.size, actx, stream);
      h->blobs[1] = alloc(bb.size, actx, stream);
      if (!h->blobs[0] || !h->blobs[1]) { st = SPTIR_ERR_ALLOC; goto fail; }
      h->device_bytes += ba.size + bb.size;
      char* a0 = (char*)h->blobs[0];
      char* b0 = (char*)h->blobs[1];
      h->bucket_row_ptr = (int64_t*)(a0 + a_row_ptr); h->bucket_slot_ptr = (int64_t*)(a0 + a_slot_ptr);
      h->rem_part_ptr = (int32_t*)(a0 + a_rem_part); h->rem_ptr = (int64_t*)(a0 + a_rem_ptr);
      h->row_ids = (int32_t*)(a0 + a_row_ids); h->row_len = (int32_t*)(a0 + a_row_len);
      h->rb_chunk_ptr = (int64_t*)(a0 + a_rb_chunk);
      if (one_value_per_row) h->row_val = (float*)(a0 + a_row_val);
      if (want_heavy) h->row_slot_ptr = (int32_t*)(a0 + a_row_slot);
      h->cols = (int32_t*)(b0 + b_cols); h->vals = (float*)(b0 + b_vals);
      h->canonical_bytes = bb.size;
    }
    if (one_value_per_row) {
      hipLaunchKernelGGL(k_row_values, dim3((unsigned)((s.n_rows + 255) / 256)), dim3(256), 0, stream, s.n_rows,
                         csr->indptr, csr->values, h->row_val);
      BUILD_HIP(hipGetLastError());
    }
    BUILD_HIP(hipMemcpyAsync(h->bucket_row_ptr, row_ptr, sizeof(int64_t) * (B + 1), hipMemcpyHostToDevice, stream));
    BUILD_HIP(hipMemcpyAsync(h->bucket_slot_ptr, slot_ptr, sizeof(int64_t) * (B + 1), hipMemcpyHostToDevice, stream));
    BUILD_HIP(hipMemcpyAsync(h->rem_part_ptr, rem_part_ptr, sizeof(int32_t) * (s.c + 1), hipMemcpyHostToDevice, stream));
    BUILD_HIP(hipMemcpyAsync(d_rnnz_base, rnnz_base, sizeof(int64_t) * s.c, hipMemcpyHostToDevice, stream));

    // ---- stable scatter
    if (s.NB > 0) {
      ScatterArgs a;
      a.indptr = csr->indptr; a.indices = csr->indices; a.values = csr->values;
      a.bound = d_bound; a.counts = d_counts; a.rem_nnz = d_rnnz;
      a.bucket_row_ptr = h->bucket_row_ptr; a.bucket_slot_ptr = h->bucket_slot_ptr;
      a.rem_part_ptr = h->rem_part_ptr; a.rem_nnz_base = d_rnnz_base;
      a.row_ids = h->row_ids; a.cols = h->cols; a.vals = h->vals; a.rem_ptr = h->rem_ptr; a.row_len = h->row_len;
      a.piece_of = d_piece_of;
      a.R = h->R; a.S = h->S; a.M = M; a.T = T;
      hipLaunchKernelGGL(k_scatter, dim3((unsigned)n_pair_blocks), dim3(kBuildBlock), 0, stream, s, a);
    } else {
      int64_t* zero = (int64_t*)(host.base + h_misc + 8);
      *zero = 0;
      BUILD_HIP(hipMemcpyAsync(h->rem_ptr, zero, sizeof(int64_t), hipMemcpyHostToDevice, stream));
      BUILD_HIP(hipMemsetAsync(h->row_ids + h->R + M, 0, sizeof(int32_t) * kChunkSlots, stream));
      BUILD_HIP(hipMemsetAsync(h->cols + h->S + T, 0, sizeof(int32_t) * kChunkSlots, stream));
      BUILD_HIP(hipMemsetAsync(h->vals + h->S + T, 0, sizeof(float) * kChunkSlots, stream));
    }
    BUILD_HIP(hipGetLastError());

    // ---- heavy pieces: how many, and how many chunks (prefixes over the pieces in row_ids order)
    BUILD_HIP(hipMemsetAsync(d_totals, 0, o_nnz_slots - o_totals + sizeof(long long) * kFlagSlots * kFlagStride, stream));
    if (want_heavy) {
      hipLaunchKernelGGL(k_heavy_counts, dim3((unsigned)((n_pieces + 256) / 256)), dim3(256), 0, stream, n_pieces,
                         h->row_len, cs.long_len, d_unit, d_hent, (unsigned long long*)d_nnz_slots);
      BUILD_HIP(hipGetLastError());
      st = device_exclusive_scan(d_unit, n_pieces + 1, d_seq_base, stream);
      if (st != SPTIR_OK) goto fail;
      st = device_exclusive_scan(d_hent, n_pieces + 1, d_seq_base, stream);
      if (st != SPTIR_OK) goto fail;
    }

    // ---- chunk descriptors of the lists, grouped by (phase, row block)
    if (n_cells > 0) {
      BUILD_HIP(hipMemsetAsync(d_group_tot, 0, sizeof(long long) * (size_t)n_seq * kGroupSeq, stream));
      hipLaunchKernelGGL(k_cell_bounds, dim3((unsigned)((n_bounds + 255) / 256)), dim3(256), 0, stream, cs,
                         h->bucket_row_ptr, h->rem_part_ptr, h->row_ids, d_bounds);
      hipLaunchKernelGGL(k_part_chunk_counts, dim3((unsigned)((n_parts + 255) / 256)), dim3(256), 0, stream, cs,
                         n_parts, d_bounds, h->row_len, d_cell_chunks);
      hipLaunchKernelGGL(k_group_scan, dim3((unsigned)((n_groups + 3) / 4)), dim3(256), 0, stream, cs, n_groups,
                         d_cell_chunks, d_group_tot, (unsigned long long*)(d_nnz_slots + 1));
      // chunks before a cell = its prefix inside the group + the group's inside its sequence + the sequence's
      hipLaunchKernelGGL(k_scan_sequences<long long>, dim3((unsigned)n_seq), dim3(kBuildBlock), 0, stream,
                         d_group_tot, (int32_t)kGroupSeq, d_seq_tot);
      hipLaunchKernelGGL(k_scan_sequences<long long>, dim3(1), dim3(kBuildBlock), 0, stream, d_seq_tot,
                         (int32_t)n_seq, d_totals);
      BUILD_HIP(hipGetLastError());
    }
    // one report for the host: the totals
    {
      hipLaunchKernelGGL(k_report, dim3(1), dim3(64), 0, stream, d_totals, d_nnz_slots,
                         want_heavy ? d_unit : nullptr, want_heavy ? d_hent : nullptr, n_pieces, d_report2);
      BUILD_HIP(hipGetLastError());
      BUILD_HIP(hipMemcpyAsync(host.base + h_report2, d_report2, sizeof(long long) * report2_count,
                               hipMemcpyDeviceToHost, stream));
    }
    // (the GPU is busy: the allocations whose sizes are known come now)
    if (with_spmm_plan) {
      const size_t bytes = sizeof(PiecePlace) * (size_t)(n_pieces ? n_pieces : 1);
      tmp_place = scratch_alloc(bytes, alloc, actx, stream);
      if (!tmp_place) { st = SPTIR_ERR_ALLOC; goto fail; }
      BUILD_HIP(hipMemsetAsync(tmp_place, 0, bytes, stream));  // len 0: not queued
    }
    BUILD_HIP(hipStreamSynchronize(stream));
    const long long* report2 = (const long long*)(host.base + h_report2);
    const long long n_chunks = report2[0];
    h->n_heavy_nnz = report2[1];
    const int64_t max_list_len = report2[4];
    // the lists' chunks come first in the stream (each list a whole number of quads), then the heavy chunks
    // (report2[3]: slots of the heavy sequence)
    const int64_t n_heavy_chunks = (chunks_of_slots(report2[3]) + kChunksPerQuad - 1) / kChunksPerQuad * kChunksPerQuad;
    h->n_chunks = n_chunks;
    h->n_heavy = report2[2];
    h->heavy_chunk0 = n_chunks;
    h->n_heavy_chunks = n_heavy_chunks;
    // Chunks per heavy list: 16 where that still gives thousands of lists; a graph with few heavy chunks gets
    // shorter lists, or its heavy launch would be a handful of wavefronts walking 16 chunks each while the GPU idles.
    int32_t list_chunks = kHeavyListChunks;
    while (list_chunks > kChunksPerQuad && n_heavy_chunks / list_chunks < 4096) list_chunks /= 2;
    h->heavy_list_chunks = list_chunks;
    h->n_heavy_lists = (int32_t)((n_heavy_chunks + list_chunks - 1) / list_chunks);
    h->n_partial_rows = h->n_heavy + h->n_heavy_lists;
    if (h->n_heavy == 0) h->row_slot_ptr = nullptr;  // (its room in the first allocation stays unused)
    const int64_t all_chunks = n_chunks + n_heavy_chunks;
    if (h->n_partial_rows > 0x7FFFFFFF || all_chunks > 0x7FFFFFFF) { st = SPTIR_ERR_OVERFLOW; goto fail; }
    const int32_t n_units = (int32_t)h->n_heavy;
    int64_t* unit_slot0 = nullptr;
    int32_t *unit_start = nullptr, *unit_end = nullptr, *quad_unit = nullptr;
    // ---- the arrays of the SpMM plan, one allocation; the temporaries of this stage, another.  A row of Y takes
    // one partial-sum row per heavy piece it has plus one per list boundary such a piece crosses, so there are at
    // most n_partial_rows of them; the rows with heavy pieces are at most as many as there are such pieces.
    {
      Blob bc, bt;
      const bool heavy = h->n_heavy > 0;
      const size_t c_first_slot = bc.reserve(heavy ? sizeof(int32_t) * (size_t)h->n_heavy_lists : 0);
      const size_t c_row_slots = bc.reserve(heavy ? sizeof(int32_t) * (size_t)h->n_partial_rows : 0);
      const size_t c_heavy_rows = bc.reserve(heavy ? sizeof(int32_t) * (size_t)std::min<int64_t>(s.n_rows, h->n_heavy) : 0);
      const size_t c_rb_order = bc.reserve(sizeof(int32_t) * (size_t)(n_groups ? n_groups : 1));
      const size_t c_stream = bc.reserve(sizeof(int32_t) * ((h->compact_stream ? 2 : 3) - (one_value_per_row ? 1 : 0)) *
                                         kChunkSlots * (size_t)(all_chunks ? all_chunks : 1));
      const size_t c_partial = bc.reserve(heavy ? sizeof(float) * kPartialFeat * (size_t)h->n_partial_rows : 0);
      const size_t t_chunks = bt.reserve(sizeof(Chunk) * (size_t)(n_chunks ? n_chunks : 1));
      const size_t t_slot0 = bt.reserve(heavy ? sizeof(int64_t) * (size_t)n_units : 0);
      const size_t t_start = bt.reserve(heavy ? sizeof(int32_t) * ((size_t)n_units + 1) : 0);
      const size_t t_end = bt.reserve(heavy ? sizeof(int32_t) * (size_t)n_units : 0);
      const size_t t_quad = bt.reserve(heavy ? sizeof(int32_t) * (size_t)(n_heavy_chunks / kChunksPerQuad + 1) : 0);
      h->blobs[2] = alloc(bc.size, actx, stream);
      tmp_chunks = scratch_alloc(bt.size, alloc, actx, stream);
      if (!h->blobs[2] || !tmp_chunks) { st = SPTIR_ERR_ALLOC; goto fail; }
      h->device_bytes += bc.size;
      char* c0 = (char*)h->blobs[2];
      char* t0 = (char*)tmp_chunks;
      if (heavy) {
        h->hlist_first_slot = (int32_t*)(c0 + c_first_slot); h->row_slots = (int32_t*)(c0 + c_row_slots);
        h->heavy_rows = (int32_t*)(c0 + c_heavy_rows); h->partial = (float*)(c0 + c_partial);
        unit_slot0 = (int64_t*)(t0 + t_slot0); unit_start = (int32_t*)(t0 + t_start);
        unit_end = (int32_t*)(t0 + t_end); quad_unit = (int32_t*)(t0 + t_quad);
      }
      if (n_groups > 0) h->rb_order = (int32_t*)(c0 + c_rb_order);
      h->stream = (int32_t*)(c0 + c_stream);
      (void)t_chunks;  // (offset 0)
      BUILD_HIP(hipMemsetAsync(tmp_chunks, 0, sizeof(Chunk) * (size_t)(n_chunks ? n_chunks : 1), stream));  // count 0 marks the padding chunks
    }
    if (h->n_heavy > 0) {
      // ---- heavy pieces: where every piece lies, the first partial-sum row of every heavy list, which
      // partial-sum rows each row of Y takes
      hipLaunchKernelGGL(k_heavy_units, dim3((unsigned)((n_pieces + 256) / 256)), dim3(256), 0, stream, n_pieces,
                         h->row_len, d_unit, d_hent, B, s.k, h->R, h->S, h->bucket_row_ptr, h->bucket_slot_ptr,
                         h->rem_ptr, cs.long_len, unit_start, unit_end, unit_slot0, quad_unit);
      hipLaunchKernelGGL(k_heavy_list_slots, dim3((unsigned)((h->n_heavy_lists + 255) / 256)), dim3(256), 0, stream,
                         h->n_heavy_lists, list_chunks, n_units, unit_end, h->hlist_first_slot);
      hipLaunchKernelGGL(k_row_slot_counts, dim3((unsigned)((s.n_rows + 256) / 256)), dim3(256), 0, stream, s.n_rows,
                         s.c, list_chunks, d_piece_of, h->row_len, d_unit, d_hent, h->row_slot_ptr);
      BUILD_HIP(hipGetLastError());
      st = device_exclusive_scan(h->row_slot_ptr, (int64_t)s.n_rows + 1, d_seq_base, stream);
      if (st != SPTIR_OK) goto fail;
      // the rows that have heavy pieces, compacted: the launch that adds their partial sums to Y visits only them
      hipLaunchKernelGGL(k_heavy_row_flags, dim3((unsigned)((s.n_rows + 256) / 256)), dim3(256), 0, stream, s.n_rows,
                         h->row_slot_ptr, d_row_flags);
      BUILD_HIP(hipGetLastError());
      st = device_exclusive_scan(d_row_flags, (int64_t)s.n_rows + 1, d_seq_base, stream);
      if (st != SPTIR_OK) goto fail;
      hipLaunchKernelGGL(k_row_slot_fill, dim3((unsigned)((s.n_rows + 255) / 256)), dim3(256), 0, stream, s.n_rows,
                         s.c, list_chunks, d_piece_of, h->row_len, d_unit, d_hent, h->row_slot_ptr, h->row_slots);
      hipLaunchKernelGGL(k_heavy_row_fill, dim3((unsigned)((s.n_rows + 255) / 256)), dim3(256), 0, stream, s.n_rows,
                         h->row_slot_ptr, d_row_flags, h->heavy_rows);
      hipLaunchKernelGGL(k_pick2, dim3(1), dim3(64), 0, stream, h->row_slot_ptr + s.n_rows,
                         d_row_flags + s.n_rows, d_report3);
      BUILD_HIP(hipGetLastError());
      BUILD_HIP(hipMemcpyAsync(host.base + h_report3, d_report3, sizeof(int32_t) * 2, hipMemcpyDeviceToHost, stream));
    }
    StreamShape ss;
    ss.stream = h->stream; ss.compact = h->compact_stream; ss.log2_rb = cs.log2_rb; ss.unit = h->row_val ? 1 : 0;
    ss.phase_width = (int32_t)((int64_t)cs.ppg * s.w > 0x7FFFFFFF ? 0x7FFFFFFF : (int64_t)cs.ppg * s.w);
    if (n_parts > 0)
      hipLaunchKernelGGL(k_part_fill_chunks, dim3((unsigned)((n_parts + 255) / 256)), dim3(256), 0, stream, cs, ss,
                         n_parts, d_bounds, d_cell_chunks, d_group_tot, d_seq_tot, h->row_len, h->row_ids,
                         h->bucket_row_ptr, h->bucket_slot_ptr, h->rem_ptr, h->S, (Chunk*)tmp_chunks,
                         (PiecePlace*)tmp_place, h->rb_chunk_ptr, (int64_t)n_chunks);
    if (h->n_heavy > 0)
      hipLaunchKernelGGL(k_pack_heavy, dim3((unsigned)((n_heavy_chunks / kPackRun + 3) / 4)), dim3(256), 0, stream,
                         n_heavy_chunks, (int64_t)n_chunks, ss, n_units, unit_start, unit_end, unit_slot0, quad_unit,
                         h->cols, h->vals);
    if (n_chunks > 0) {
      int64_t blocks = (n_chunks + 3) / 4;
      if (blocks > 0x7FFFFFFF) { st = SPTIR_ERR_OVERFLOW; goto fail; }
      hipLaunchKernelGGL(k_pack_stream, dim3((unsigned)blocks), dim3(256), 0, stream, (int64_t)n_chunks, ss,
                         (const Chunk*)tmp_chunks, h->row_ids, h->cols, h->vals);
      if (n_pieces > 0)
        hipLaunchKernelGGL(k_pack_pieces, dim3((unsigned)((n_pieces + 255) / 256)), dim3(256), 0, stream, n_pieces, ss,
                           (const PiecePlace*)tmp_place, h->row_ids, h->cols, h->vals);
    }
    BUILD_HIP(hipGetLastError());
    if (n_parts == 0) {  // no lists: the one element of rb_chunk_ptr
      int64_t* zero = (int64_t*)(host.base + h_misc + 16);
      *zero = 0;
      BUILD_HIP(hipMemcpyAsync(h->rb_chunk_ptr, zero, sizeof(int64_t), hipMemcpyHostToDevice, stream));
    }
    if (n_groups > 0) {
      // ---- launch order of the row blocks: longest list first
      st = order_row_blocks(h->rb_chunk_ptr, cs.n_phases, cs.n_rb, max_list_len, h->rb_order, alloc, free_, actx,
                            stream, &tmp_order);
      if (st != SPTIR_OK) goto fail;
    }
    BUILD_HIP(hipStreamSynchronize(stream));
    if (h->n_heavy > 0) {
      const int32_t* report3 = (const int32_t*)(host.base + h_report3);
      h->n_row_slots = report3[0];
      h->n_heavy_rows = report3[1];
    }
    if (opt.release_canonical && with_spmm_plan) {
      // sptir_spmm reads the stream only
      free_(h->blobs[1], actx);
      h->blobs[1] = nullptr;
      h->cols = nullptr; h->vals = nullptr;
      h->device_bytes -= h->canonical_bytes;
      h->canonical_released = 1;
    }
  }
  scratch_free(tmp.base, free_, actx);
  scratch_free(tmp2.base, free_, actx);
  scratch_free(tmp_chunks, free_, actx);
  scratch_free(tmp_place, free_, actx);
  scratch_free(tmp_order, free_, actx);
  pinned_pool().release(pinned);
  *out = h;
  return SPTIR_OK;

fail:
  (void)hipStreamSynchronize(stream);
  scratch_free(tmp.base, free_, actx);
  scratch_free(tmp2.base, free_, actx);
  scratch_free(tmp_chunks, free_, actx);
  scratch_free(tmp_place, free_, actx);
  scratch_free(tmp_order, free_, actx);
  pinned_pool().release(pinned);
  sptir_hyb_destroy(h);
  return st;
#undef BUILD_HIP
}
