// fp32 projection for the fp32 (small, parity-oriented) configuration:
// out[m][n] = sum_k X[m][k] * W[n][k], W row-major, one wavefront per output row.
#include "common.h"
#include "dart_internal.h"

namespace dart {

template <int MAXM>
__global__ __launch_bounds__(256) void gemv_f32_kernel(const float *__restrict__ W,
                                                       const float *__restrict__ X, int M, int row0,
                                                       int nrows, int Kd, float *__restrict__ out,
                                                       int out_stride) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= nrows) return;                       // whole wavefront leaves together
  const float *w = W + (size_t)(row0 + r) * Kd;
  float acc[MAXM];
#pragma unroll
  for (int m = 0; m < MAXM; ++m) acc[m] = 0.f;
  for (int k = lane * 4; k < Kd; k += 256) {    // Kd is a multiple of 4
    const float4 wv = *reinterpret_cast<const float4 *>(w + k);
#pragma unroll
    for (int m = 0; m < MAXM; ++m) {
      if (m < M) {
        const float4 xv = *reinterpret_cast<const float4 *>(X + (size_t)m * Kd + k);
        acc[m] += wv.x * xv.x + wv.y * xv.y + wv.z * xv.z + wv.w * xv.w;
      }
    }
  }
#pragma unroll
  for (int m = 0; m < MAXM; ++m) {
    if (m < M) {
      const float s = wave_sum(acc[m]);
      if (lane == 0) out[(size_t)m * out_stride + r] = s;
    }
  }
}

// Rows [row0, row0+nrows) of W; out[m][j] for j in [0, nrows).
hipError_t launch_gemv_f32(const DeviceMatrix &W, int row0, int nrows, const float *X, int M,
                           float *out, int out_stride, hipStream_t st) {
  hipLaunchKernelGGL(gemv_f32_kernel<DART_SKINNY_ROWS>, dim3((nrows + 3) / 4), dim3(256), 0, st,
                     (const float *)W.data, X, M, row0, nrows, W.Kd, out, out_stride);
  return hipGetLastError();
}

}  // namespace dart
