// Skinny projection on bf16 weights: out[m][n] = sum_k X[m][k] W[n][k] for M <= 16 rows.
//
// This is the weight-streaming step of the draft forward (QKV, O, gate/up, down and above
// all the LM head, 70 % of the bytes at Qwen3-14B shapes): every weight is read from HBM
// exactly once and used for all M rows, so the kernel is bound by the HBM stream.  At
// 8 TB/s and 256 CUs about 6.5 bf16 weights arrive per CU per clock; 8 rows of plain fp32
// FMAs per weight would need 52 of the CU's 64 non-packed FMA lanes per clock, so the
// contraction itself runs on the matrix cores (v_mfma_f32_16x16x32_bf16, fp32 accumulate),
// which leaves the vector ALUs idle and the kernel on the memory roof.
//
// Layout: weights are re-tiled once at load time so that the 1 KiB a wavefront fetches per
// MFMA (lane l: 16 contiguous bytes at tile + 16*l) is already the A operand -- 16 output
// rows x 32 inputs -- with no LDS staging or shuffles.  Tiles of one 16-row strip are
// contiguous along k, so a wavefront streams a contiguous span.
//
// Work split: a workgroup is 8 wavefronts that cut the k range of a strip 8 ways; each
// keeps its slice of the activations (B operands, fp32 split once into bf16 hi + lo parts,
// two MFMAs per weight tile) in registers for the whole kernel and walks the workgroup's
// strips.  Weight tiles go through a small rolling register buffer whose loads are issued
// right after the MFMAs that free each register (several KiB in flight per wavefront).  Per strip the 8 partial 16x16 tiles are summed through LDS in a fixed order
// (deterministic), one barrier per strip.  When the k range is too long for the register
// budget the range is cut into chunks handled by different workgroups, and the consumer
// adds the chunk partials (also in fixed order).
#include "common.h"
#include "dart_internal.h"

namespace dart {

constexpr int GEMV_WAVES = 8;
constexpr int GEMV_THREADS = GEMV_WAVES * 64;
constexpr int GEMV_KPW_MAX = 20;          // k-steps (of 32 inputs) per wavefront per chunk

int gemv_bf16_chunks(int Kd) {
  const int KT = Kd / 32;
  return (KT + GEMV_WAVES * GEMV_KPW_MAX - 1) / (GEMV_WAVES * GEMV_KPW_MAX);
}

template <int KPW, int D>
__global__ __launch_bounds__(GEMV_THREADS) void gemv_bf16_kernel(
    const uint4 *__restrict__ Wp,   // packed tiles, 64 uint4 per tile
    const float *__restrict__ X,    // [M][Kd]
    int M, int KT, int kpw, int nchunks, int strip0, int nstrips, int n_cols,
    float *__restrict__ out, int out_stride, size_t chunk_stride) {
  static_assert(KPW % D == 0, "a register of the rolling buffer must serve the same slots in every strip");
  __shared__ float part[2][GEMV_WAVES][256];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 15, gq = lane >> 4;
  const int chunk = blockIdx.x % nchunks;
  const int wg = blockIdx.x / nchunks, nwg = gridDim.x / nchunks;
  const int ks0 = (chunk * GEMV_WAVES + wave) * kpw;
  const int nk = max(0, min(kpw, KT - ks0));           // wave-uniform
  const int Kd = KT * 32;

  // B operands: activations of this wavefront's k slice, column m = lane % 16, split into
  // bf16 hi + bf16 lo (x ~= hi + lo to ~2^-17) so that activations keep fp32-like accuracy
  // while the weights stay the exact bf16 values.
  bf16x8_t bhi[KPW], blo[KPW];
#pragma unroll
  for (int t = 0; t < KPW; ++t) {
    union { bf16x8_t v; bf16_t e[8]; } h, l;
#pragma unroll
    for (int e = 0; e < 8; ++e) h.e[e] = l.e[e] = 0;
    if (t < nk && col < M) {
      const float *src = X + (size_t)col * Kd + (size_t)(ks0 + t) * 32 + 8 * gq;
      const float4 lo4 = *reinterpret_cast<const float4 *>(src);
      const float4 hi4 = *reinterpret_cast<const float4 *>(src + 4);
      const float x[8] = {lo4.x, lo4.y, lo4.z, lo4.w, hi4.x, hi4.y, hi4.z, hi4.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        h.e[e] = f32_to_bf16(x[e]);
        l.e[e] = f32_to_bf16(x[e] - bf16_to_f32(h.e[e]));
      }
    }
    bhi[t] = h.v;
    blo[t] = l.v;
  }

  // Rolling buffer of D weight tiles: register t % D serves slot t of every strip; the load
  // for its next slot is issued right after the MFMAs that free it, so about D KiB stay in
  // flight per wavefront across strip boundaries.
  union AOp { uint4 u; bf16x8_t v; };
  AOp aop[D];
  int s = wg;                                          // strip index relative to strip0
  if (s < nstrips) {
    const uint4 *tile = Wp + ((size_t)(strip0 + s) * KT + ks0) * 64 + lane;
#pragma unroll
    for (int r = 0; r < D; ++r)
      if (r < nk) aop[r].u = tile[(size_t)r * 64];
  }
  int buf = 0;
  for (; s < nstrips; s += nwg) {
    const int sn = s + nwg;
    const bool more = sn < nstrips;
    const uint4 *cur = Wp + ((size_t)(strip0 + s) * KT + ks0) * 64 + lane;
    const uint4 *next = Wp + ((size_t)(strip0 + (more ? sn : s)) * KT + ks0) * 64 + lane;
    f32x4_t acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < KPW; ++t) {
      if (t < nk) {
        acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aop[t % D].v, bhi[t], acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aop[t % D].v, blo[t], acc1, 0, 0, 0);
        if (t + D < nk)
          aop[t % D].u = cur[(size_t)(t + D) * 64];
        else if (more && (t % D) < nk)
          aop[t % D].u = next[(size_t)(t % D) * 64];
      }
    }
    *reinterpret_cast<float4 *>(&part[buf][wave][lane * 4]) =
        make_float4(acc0[0] + acc1[0], acc0[1] + acc1[1], acc0[2] + acc1[2], acc0[3] + acc1[3]);
    __syncthreads();
    if (threadIdx.x < 256) {
      const int m = threadIdx.x >> 4, row = threadIdx.x & 15;
      const int idx = (((row >> 2) * 16) + m) * 4 + (row & 3);   // D[row][m] lives in lane (row/4)*16+m, reg row%4
      float v = 0.f;
#pragma unroll
      for (int w = 0; w < GEMV_WAVES; ++w) v += part[buf][w][idx];
      const int c = s * 16 + row;
      if (m < M && c < n_cols) out[chunk * chunk_stride + (size_t)m * out_stride + c] = v;
    }
    buf ^= 1;
  }
}

// Strips [strip0, strip0+nstrips) of the packed matrix; out[chunk][m][j], j < nstrips*16
// (columns beyond W.n_real - strip0*16 are not written).
hipError_t launch_gemv_bf16(const DeviceMatrix &W, int strip0, int nstrips, const float *X, int M,
                            float *out, int out_stride, size_t chunk_stride, int *chunks,
                            hipStream_t st) {
  const int KT = W.Kd / 32;
  const int nchunks = gemv_bf16_chunks(W.Kd);
  const int kpw = (KT + GEMV_WAVES * nchunks - 1) / (GEMV_WAVES * nchunks);
  if (chunks) *chunks = nchunks;
  const int n_cols = min(nstrips * 16, W.n_real - strip0 * 16);
  int wgs = 512 / nchunks;                             // two workgroups per CU on 256 CUs
  if (wgs > nstrips) wgs = nstrips;
  if (wgs < 1) wgs = 1;
  dim3 grid(wgs * nchunks), block(GEMV_THREADS);
  const uint4 *wp = (const uint4 *)W.data;
#define DART_GEMV_LAUNCH(KPW, D)                                                                \
  hipLaunchKernelGGL((gemv_bf16_kernel<KPW, D>), grid, block, 0, st, wp, X, M, KT, kpw, nchunks,  \
                     strip0, nstrips, n_cols, out, out_stride, chunk_stride)
  if (kpw <= 4) DART_GEMV_LAUNCH(4, 4);
  else if (kpw <= 8) DART_GEMV_LAUNCH(8, 8);
  else if (kpw <= 12) DART_GEMV_LAUNCH(12, 6);
  else if (kpw <= 16) DART_GEMV_LAUNCH(16, 8);
  else DART_GEMV_LAUNCH(20, 10);
#undef DART_GEMV_LAUNCH
  return hipGetLastError();
}

}  // namespace dart
