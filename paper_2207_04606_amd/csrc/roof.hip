// Microbenchmarks of the two on-chip roofs the SpMM kernels are priced against: how fast a CU pulls 128-byte rows
// of X at random through the vector-memory path (the gather every stored non-zero costs), and how fast it issues
// float32 FMAs.  They belong to the measured product: bench.py runs them next to the SpMM timings so that the
// "binding roof" it reports is a number taken on the same GPU in the same process.
#include "sptir_internal.h"

namespace sptir {
namespace {

__device__ __forceinline__ unsigned lcg(unsigned s) { return s * 1664525u + 1013904223u; }

// Every group of 8 lanes reads one 128-byte line (lane: 16 bytes) of a random row of the window
// [0, n_rows) x [tile * 32, tile * 32 + 32) of X, 8 loads in flight per lane, like the SpMM kernels' gather step.
// The feature tile follows the workgroup id modulo 8 the way the SpMM kernels bind tiles to XCDs when
// `tiles` > 1, so that an XCD's L2 sees n_rows * 128 bytes.
__global__ __launch_bounds__(256) void k_roof_gather(const float* __restrict__ X, unsigned n_rows, int row_floats,
                                                     int tiles, int iters, float* sink) {
  const int lane = threadIdx.x & 63, g = lane >> 3, fl = lane & 7;
  const unsigned wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int tile = tiles > 1 ? (int)(blockIdx.x & 7) % tiles : 0;
  unsigned s = (wave * 8u + g) * 2654435761u + 12345u;
  const float* Xf = X + tile * 32 + fl * 4;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
    float4 x[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      s = lcg(s);
      const unsigned r = (unsigned)(((unsigned long long)(s >> 4) * n_rows) >> 28);
      x[u] = *reinterpret_cast<const float4*>(Xf + (size_t)r * row_floats);
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) { acc[0] += x[u].x; acc[1] += x[u].y; acc[2] += x[u].z; acc[3] += x[u].w; }
  }
  const float t = acc[0] + acc[1] + acc[2] + acc[3];
  if (t == 1234.5f) sink[0] = t;  // keeps the loads alive; X is zero-filled or random, the store all but never happens
}

// 8 independent FMA chains per lane, `iters` rounds of 8 FMAs each: 16 flops per lane and round
__global__ __launch_bounds__(256) void k_roof_fma(int iters, float seed, float* sink) {
  float a[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) a[i] = seed + (float)(threadIdx.x + i);
  const float m = 1.0000001f, c = 1e-7f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) a[i] = fmaf(a[i], m, c);
  }
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) t += a[i];
  if (t == 1234.5f) sink[0] = t;
}

}  // namespace
}  // namespace sptir

using namespace sptir;

extern "C" sptir_status_t sptir_roof_gather(const float* X, int64_t n_rows, int32_t row_floats, int32_t tiles,
                                            int32_t n_workgroups, int32_t iters, float* sink, void* stream_,
                                            float* ms_out, double* bytes_out) {
  if (!X || !sink || !ms_out || !bytes_out) return SPTIR_ERR_INVALID_ARG;
  if (n_rows < 1 || n_rows > 0x0FFFFFFF || row_floats < 32 || row_floats % 4 != 0 || ((uintptr_t)X & 15) != 0)
    return SPTIR_ERR_INVALID_ARG;
  if (tiles < 1 || tiles > 8 || tiles * 32 > row_floats || n_workgroups < 1 || iters < 1) return SPTIR_ERR_INVALID_ARG;
  hipStream_t stream = (hipStream_t)stream_;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  SPTIR_HIP(hipEventCreate(&e0));
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return note_hip_error(hipGetLastError(), "hipEventCreate"); }
  sptir_status_t st = SPTIR_OK;
  // one untimed launch, then the timed one
  hipLaunchKernelGGL(k_roof_gather, dim3((unsigned)n_workgroups), dim3(256), 0, stream, X, (unsigned)n_rows,
                     row_floats, tiles, iters, sink);
  if (hipEventRecord(e0, stream) != hipSuccess) st = note_hip_error(hipGetLastError(), "hipEventRecord");
  hipLaunchKernelGGL(k_roof_gather, dim3((unsigned)n_workgroups), dim3(256), 0, stream, X, (unsigned)n_rows,
                     row_floats, tiles, iters, sink);
  if (st == SPTIR_OK && (hipEventRecord(e1, stream) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                         hipEventElapsedTime(ms_out, e0, e1) != hipSuccess))
    st = note_hip_error(hipGetLastError(), "timing the gather roof");
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  // 4 wavefronts per workgroup, 8 loads of 64 lanes x 16 bytes per round
  *bytes_out = (double)n_workgroups * 4.0 * (double)iters * 8.0 * 1024.0;
  return st;
}

extern "C" sptir_status_t sptir_roof_fma(int32_t n_workgroups, int32_t iters, float* sink, void* stream_,
                                         float* ms_out, double* flops_out) {
  if (!sink || !ms_out || !flops_out || n_workgroups < 1 || iters < 1) return SPTIR_ERR_INVALID_ARG;
  hipStream_t stream = (hipStream_t)stream_;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  SPTIR_HIP(hipEventCreate(&e0));
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return note_hip_error(hipGetLastError(), "hipEventCreate"); }
  sptir_status_t st = SPTIR_OK;
  hipLaunchKernelGGL(k_roof_fma, dim3((unsigned)n_workgroups), dim3(256), 0, stream, iters, 1.0f, sink);
  if (hipEventRecord(e0, stream) != hipSuccess) st = note_hip_error(hipGetLastError(), "hipEventRecord");
  hipLaunchKernelGGL(k_roof_fma, dim3((unsigned)n_workgroups), dim3(256), 0, stream, iters, 1.0f, sink);
  if (st == SPTIR_OK && (hipEventRecord(e1, stream) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                         hipEventElapsedTime(ms_out, e0, e1) != hipSuccess))
    st = note_hip_error(hipGetLastError(), "timing the FMA roof");
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  *flops_out = (double)n_workgroups * 256.0 * (double)iters * 16.0;
  return st;
}
