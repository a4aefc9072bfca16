// Device helpers shared by the kernels of the DART drafting step (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint16_t bf16_t;  // raw bfloat16 bit pattern

typedef _Float16 f16_t;

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

#define DART_WAVE 64

__device__ __forceinline__ float bf16_to_f32(bf16_t b) {
  return __uint_as_float(((uint32_t)b) << 16);
}

// round-to-nearest-even; inputs are finite on this path
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return bf16_to_f32(v); }
__device__ __forceinline__ float to_f32(f16_t v) { return (float)v; }

template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return f32_to_bf16(v); }
// fp16 (round-to-nearest-even), saturating at the largest finite value instead of overflowing
template <> __device__ __forceinline__ f16_t from_f32<f16_t>(float v) {
  return (f16_t)fminf(fmaxf(v, -65504.0f), 65504.0f);
}

// Wavefront-wide max of an unsigned 32-bit value on the DPP data path (row shifts, then the
// gfx9 row broadcasts), result returned to every lane.  Lanes without a DPP source read 0,
// which is neutral for an unsigned max, and max is idempotent, so overlapping shifts are fine.
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, false));  // row_shr:1
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, false));  // row_shr:2
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, false));  // row_shr:4
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, false));  // row_shr:8
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xf, 0xf, false));  // row_bcast:15
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xf, 0xf, false));  // row_bcast:31
  return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// Wavefront-wide max of a 64-bit key: max of the high words, then max of the low words among
// the lanes that hold that high word.
// Wavefront-wide float sum / max and integer inclusive prefix sum on the DPP data path: row
// shifts by 1, 2, 4, 8 build an inclusive scan inside each row of 16 lanes (a lane without a
// source takes the identity), row_bcast:15 into rows 1 and 3 and row_bcast:31 into rows 2 and 3
// extend it over the wavefront; lane 63 then holds the total.  A few cycles per step, where the
// __shfl forms go through the LDS crossbar.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_f32(float identity, float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(identity), __float_as_int(v), CTRL,
                                                     ROW_MASK, 0xf, false));
}
__device__ __forceinline__ float wave_sum_dpp(float v) {
  v += dpp_f32<0x111, 0xf>(0.f, v);
  v += dpp_f32<0x112, 0xf>(0.f, v);
  v += dpp_f32<0x114, 0xf>(0.f, v);
  v += dpp_f32<0x118, 0xf>(0.f, v);
  v += dpp_f32<0x142, 0xa>(0.f, v);
  v += dpp_f32<0x143, 0xc>(0.f, v);
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ float wave_max_dpp(float v) {
  const float lo = -3.0e38f;
  v = fmaxf(v, dpp_f32<0x111, 0xf>(lo, v));
  v = fmaxf(v, dpp_f32<0x112, 0xf>(lo, v));
  v = fmaxf(v, dpp_f32<0x114, 0xf>(lo, v));
  v = fmaxf(v, dpp_f32<0x118, 0xf>(lo, v));
  v = fmaxf(v, dpp_f32<0x142, 0xa>(lo, v));
  v = fmaxf(v, dpp_f32<0x143, 0xc>(lo, v));
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ float wave_sum(float v) { return wave_sum_dpp(v); }
__device__ __forceinline__ float wave_max(float v) { return wave_max_dpp(v); }   // values >= -3e38
// Inclusive prefix sum over the lanes (lane i: sum of lanes 0..i).
__device__ __forceinline__ int wave_scan_add_dpp(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);
  v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);
  v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);
  return v;
}

// x of this lane and of lane ^ 16 (lane ^ 32), as the two values of every lane, on the VALU:
// v_permlane16_swap exchanges the odd rows of 16 lanes of its first operand with the even rows
// of its second, v_permlane32_swap the upper half of the first with the lower half of the
// second; with both operands equal to x the two results hold x[lane & ~16] and x[lane | 16]
// (x[lane & 31] and x[lane | 32]).  The __shfl_xor forms go through the LDS instead, behind
// whatever else is queued there.
__device__ __forceinline__ void xor16_pair(float x, float &a, float &b) {
  const unsigned u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  a = __uint_as_float(r[0]);
  b = __uint_as_float(r[1]);
}
__device__ __forceinline__ void xor32_pair(float x, float &a, float &b) {
  const unsigned u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  a = __uint_as_float(r[0]);
  b = __uint_as_float(r[1]);
}
// max / sum over the four lanes l, l ^ 16, l ^ 32, l ^ 48 (the same value in all four)
__device__ __forceinline__ float quad16_max(float x) {
  float a, b;
  xor16_pair(x, a, b);
  x = fmaxf(a, b);
  xor32_pair(x, a, b);
  return fmaxf(a, b);
}
__device__ __forceinline__ float quad16_sum(float x) {
  float a, b;
  xor16_pair(x, a, b);
  x = a + b;
  xor32_pair(x, a, b);
  return a + b;
}

__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v) {
  const uint32_t hi = (uint32_t)(v >> 32);
  const uint32_t mh = wave_max_u32(hi);
  const uint32_t ml = wave_max_u32(hi == mh ? (uint32_t)v : 0u);
  return ((uint64_t)mh << 32) | ml;
}

// Packed activations of the multi-row projection, two formats:
//   terms = 2: [k-step][row tile][hi, lo][64 lanes][8 bf16], x ~= hi + lo (to 2^-17);
//   terms = 1: [k-step][row tile][64 lanes][8 fp16], saturated at the fp16 maximum.
// Lane l of a tile holds inputs 8*(l/16)..+7 of row l%16 (the B operand of the 16x16x32 MFMA).
// Eight consecutive inputs c..c+7 (c % 8 == 0) of row r are one lane's 16 bytes of a tile.
__device__ __forceinline__ uint16_t f32_to_f16_sat_bits(float x) {
  const f16_t h = (f16_t)fminf(fmaxf(x, -65504.f), 65504.f);
  return __builtin_bit_cast(uint16_t, h);
}
__device__ __forceinline__ void pack_store8(uint4 *pack, int ntiles, int terms, int r, int c,
                                            const float *x) {
  uint4 *dst = pack + ((size_t)(c >> 5) * ntiles + (r >> 4)) * (64 * terms) +
               (((c & 31) >> 3) * 16 + (r & 15));
  if (terms == 1) {
    uint32_t h[4];
#pragma unroll
    for (int e = 0; e < 4; ++e)
      h[e] = (uint32_t)f32_to_f16_sat_bits(x[2 * e]) | ((uint32_t)f32_to_f16_sat_bits(x[2 * e + 1]) << 16);
    dst[0] = make_uint4(h[0], h[1], h[2], h[3]);
    return;
  }
  uint32_t h[4], l[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const bf16_t h0 = f32_to_bf16(x[2 * e]), h1 = f32_to_bf16(x[2 * e + 1]);
    const bf16_t l0 = f32_to_bf16(x[2 * e] - bf16_to_f32(h0));
    const bf16_t l1 = f32_to_bf16(x[2 * e + 1] - bf16_to_f32(h1));
    h[e] = (uint32_t)h0 | ((uint32_t)h1 << 16);
    l[e] = (uint32_t)l0 | ((uint32_t)l1 << 16);
  }
  dst[0] = make_uint4(h[0], h[1], h[2], h[3]);
  dst[64] = make_uint4(l[0], l[1], l[2], l[3]);
}
__device__ __forceinline__ void pack_zero8(uint4 *pack, int ntiles, int terms, int r, int c) {
  uint4 *dst = pack + ((size_t)(c >> 5) * ntiles + (r >> 4)) * (64 * terms) +
               (((c & 31) >> 3) * 16 + (r & 15));
  dst[0] = make_uint4(0, 0, 0, 0);
  if (terms == 2) dst[64] = make_uint4(0, 0, 0, 0);
}

// Block-wide sum / max for blocks of up to 1024 threads; `red` is >= 16 floats of LDS.
// All threads must call; the result is returned to every thread.
__device__ __forceinline__ float block_sum(float v, float *red) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  v = wave_sum(v);
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  float t = 0.f;
  for (int w = 0; w < nw; ++w) t += red[w];
  return t;
}

__device__ __forceinline__ float block_max(float v, float *red) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  v = wave_max(v);
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  float t = red[0];
  for (int w = 1; w < nw; ++w) t = fmaxf(t, red[w]);
  return t;
}

// Monotone map float -> uint32 (larger float <=> larger key); -0 is folded into +0.
__device__ __forceinline__ uint32_t f32_sortable(float f) {
  f = f + 0.0f;
  uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float f32_unsortable(uint32_t k) {
  uint32_t u = (k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k;
  return __uint_as_float(u);
}
