// Diagnostics (include/dart_debug.h): a plain streaming read of a device buffer, the yardstick
// the weight-streaming kernels are measured against on the same GPU in the same run.
#include "common.h"
#include "dart_internal.h"

namespace dart {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

// Every lane reads 16 bytes per step, 8 independent steps in flight, non-temporal (the buffer is
// read once), a fixed span per workgroup so that each one walks a contiguous region like the
// projection kernels do.  The xor of everything read is stored only if it equals a value that
// the caller chooses so that it practically never does: the loads cannot be optimised away and
// the kernel writes nothing.
constexpr int STREAM_THREADS = 512;
constexpr int STREAM_UNROLL = 8;
template <bool NT>
__device__ __forceinline__ u32x4_t stream_load(const u32x4_t *p) {
  if constexpr (NT) return __builtin_nontemporal_load(p);
  else return *p;
}

template <bool NT>
__global__ __launch_bounds__(STREAM_THREADS) void stream_read_kernel(const u32x4_t *__restrict__ src,
                                                                     size_t n16, uint32_t never,
                                                                     uint32_t *__restrict__ sink) {
  const size_t per_wg = (n16 + gridDim.x - 1) / gridDim.x;
  const size_t begin = per_wg * blockIdx.x, end = min(n16, begin + per_wg);
  u32x4_t acc = {0, 0, 0, 0};
  size_t i = begin + threadIdx.x;
  for (; i + (size_t)(STREAM_UNROLL - 1) * STREAM_THREADS < end; i += (size_t)STREAM_UNROLL * STREAM_THREADS) {
    u32x4_t v[STREAM_UNROLL];
#pragma unroll
    for (int u = 0; u < STREAM_UNROLL; ++u) v[u] = stream_load<NT>(src + i + (size_t)u * STREAM_THREADS);
#pragma unroll
    for (int u = 0; u < STREAM_UNROLL; ++u) acc ^= v[u];
  }
  for (; i < end; i += STREAM_THREADS) acc ^= stream_load<NT>(src + i);
  const uint32_t x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
  if (x == never && sink) sink[0] = x;
}

}  // namespace dart

extern "C" dart_status dart_debug_stream_read(const void *buf, int64_t bytes, int workgroups,
                                              int non_temporal, void *sink, void *stream) {
  if (!buf || bytes < 16 || workgroups < 1 || workgroups > 65536) return DART_ERR_ARG;
  if (reinterpret_cast<uintptr_t>(buf) & 15) return DART_ERR_ARG;
  if (non_temporal)
    hipLaunchKernelGGL(dart::stream_read_kernel<true>, dim3(workgroups), dim3(dart::STREAM_THREADS), 0,
                       (hipStream_t)stream, (const dart::u32x4_t *)buf, (size_t)(bytes / 16),
                       0x9E3779B9u, (uint32_t *)sink);
  else
    hipLaunchKernelGGL(dart::stream_read_kernel<false>, dim3(workgroups), dim3(dart::STREAM_THREADS), 0,
                       (hipStream_t)stream, (const dart::u32x4_t *)buf, (size_t)(bytes / 16),
                       0x9E3779B9u, (uint32_t *)sink);
  return hipGetLastError() == hipSuccess ? DART_OK : DART_ERR_HIP;
}
