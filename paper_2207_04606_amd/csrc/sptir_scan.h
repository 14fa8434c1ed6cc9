// Device helpers shared by the builder kernels: workgroup scans and the lower
// bound in a sorted row.  Everything here has internal linkage.
#ifndef SPTIR_SCAN_H_
#define SPTIR_SCAN_H_

#include "sptir_internal.h"

namespace sptir {
namespace {

constexpr int kWaves = kBuildBlock / 64;

// first position q in [lo, hi) whose column is >= bound
__device__ __forceinline__ int lower_bound_col(const int32_t* __restrict__ indices, int lo, int hi, int64_t bound) {
  while (lo < hi) {
    int mid = lo + ((hi - lo) >> 1);
    if ((int64_t)indices[mid] < bound) lo = mid + 1; else hi = mid;
  }
  return lo;
}

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
// prefix, totals[seq] its sum.  A thread scans kScanPerThread consecutive
// elements itself, so a long sequence costs few workgroup-wide steps.
constexpr int kScanPerThread = 8;

template <typename T>
__global__ __launch_bounds__(kBuildBlock) void k_scan_sequences(T* data, int32_t len, T* totals) {
  __shared__ T wave_sums[kWaves];
  T* seq = data + (int64_t)blockIdx.x * len;
  T carry = 0;
  for (int64_t base = 0; base < len; base += (int64_t)kBuildBlock * kScanPerThread) {
    const int64_t e0 = base + (int64_t)threadIdx.x * kScanPerThread;
    T v[kScanPerThread];
    T mine = 0;
#pragma unroll
    for (int i = 0; i < kScanPerThread; ++i) {
      v[i] = (e0 + i < len) ? seq[e0 + i] : (T)0;
      mine += v[i];
    }
    T tot;
    T before = carry + block_exclusive_scan(mine, wave_sums, &tot);
#pragma unroll
    for (int i = 0; i < kScanPerThread; ++i) {
      if (e0 + i < len) seq[e0 + i] = before;
      before += v[i];
    }
    carry += tot;
  }
  if (threadIdx.x == 0) totals[blockIdx.x] = carry;
}

}  // namespace
}  // namespace sptir

#endif  // SPTIR_SCAN_H_
