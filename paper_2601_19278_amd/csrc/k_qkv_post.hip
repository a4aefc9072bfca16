// After the fused Q/K/V projection: per-head RMSNorm of q and k (optional), rotary
// positions, and the append of the new K/V rows to the draft layer's K/V buffers.
// The draft is a single layer (paper Sec. 3.2), so K/V of a row depend on that row only and
// can be kept across draft-verify iterations.
#include "common.h"
#include "dart_internal.h"

namespace dart {

// grid (pass rows, Hq + 2*Hkv heads), block = head_dim threads.
// Pass row i is position pos of sequence b (SeqBatch); q is produced for query rows only and
// stored at the compact index b*K + j; k and v of every row go to the sequence's K/V slot.
// T: storage type of the norm gains; CT: element type of q and of the K/V buffers.
template <typename T, typename CT>
__global__ __launch_bounds__(128) void qkv_post_kernel(
    SeqBatch sb, const float *__restrict__ qkv, int chunks, size_t chunk_stride, int row_stride,
    int col0, int Hq, int Hkv, int hd, int qk_norm, float eps, const T *__restrict__ q_gain,
    const T *__restrict__ k_gain, const float *__restrict__ cos_tab,
    const float *__restrict__ sin_tab, CT *__restrict__ q_out, CT *__restrict__ kbuf,
    CT *__restrict__ vbuf, size_t slot_elems, int t_cap, int tiled) {
  __shared__ float red[16];
  __shared__ float sh[128];
  const int i = blockIdx.x, hh = blockIdx.y, t = threadIdx.x;
  int b, pos, qi;
  seq_of_row(sb, i, b, pos, qi);
  const bool is_q = hh < Hq, is_k = !is_q && hh < Hq + Hkv;
  if (is_q && qi < 0) return;                     // non-query rows need no q (uniform per block)
  kbuf += (size_t)sb.slot[b] * slot_elems;
  vbuf += (size_t)sb.slot[b] * slot_elems;
  const int col = hh * hd + t - col0;             // q heads, then k heads, then v heads
  // chunk partials: up to 8 loads in flight, added in index order
  float x = 0.f;
  const float *src = qkv + (size_t)i * row_stride + col;
  for (int c0 = 0; c0 < chunks; c0 += 8) {
    float p[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) p[u] = c0 + u < chunks ? src[(size_t)(c0 + u) * chunk_stride] : 0.f;
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (c0 + u < chunks) x += p[u];
  }

  if (!is_q && !is_k) {                           // value head: store as is
    const int g = hh - Hq - Hkv;
    if (tiled)
      vbuf[(size_t)g * hd * t_cap + attn_vt_index(pos, t, hd)] = from_f32<CT>(x);
    else
      vbuf[((size_t)g * t_cap + pos) * hd + t] = from_f32<CT>(x);
    return;
  }
  if (qk_norm) {
    const float ss = block_sum(x * x, red);
    x = x * (1.0f / sqrtf(ss / (float)hd + eps)) * to_f32((is_q ? q_gain : k_gain)[t]);
  }
  sh[t] = x;
  __syncthreads();
  const int half = hd >> 1;
  const int fi = t < half ? t : t - half;
  const float c = cos_tab[(size_t)pos * half + fi], s = sin_tab[(size_t)pos * half + fi];
  const float y = t < half ? x * c - sh[t + half] * s : x * c + sh[t - half] * s;
  if (is_q) {
    q_out[((size_t)(b * sb.K + qi) * Hq + hh) * hd + t] = from_f32<CT>(y);
  } else {
    const int g = hh - Hq;
    if (tiled)
      kbuf[(size_t)g * hd * t_cap + attn_k_index(pos, t, hd)] = from_f32<CT>(y);
    else
      kbuf[((size_t)g * t_cap + pos) * hd + t] = from_f32<CT>(y);
  }
}

hipError_t launch_qkv_post(const dart_ctx *c, const SeqBatch &sb, const float *qkv, int chunks,
                           size_t chunk_stride, int row_stride, int col0, hipStream_t st) {
  const dart_config &g = c->cfg;
  const int Hq = g.n_q_heads, Hkv = g.n_kv_heads, hd = g.head_dim;
  const size_t slot_elems = (size_t)Hkv * c->t_cap * hd;
  dim3 grid(sb.row_off[sb.B], Hq + 2 * Hkv), block(hd);
  if (g.dtype == DART_BF16) {
    hipLaunchKernelGGL((qkv_post_kernel<bf16_t, f16_t>), grid, block, 0, st, sb, qkv, chunks,
                       chunk_stride, row_stride, col0, Hq, Hkv, hd, g.qk_norm, g.rms_eps,
                       (const bf16_t *)c->g_q, (const bf16_t *)c->g_k, c->rope_cos, c->rope_sin,
                       (f16_t *)c->qrot, (f16_t *)c->kbuf, (f16_t *)c->vbuf, slot_elems, c->t_cap, 1);
  } else {
    hipLaunchKernelGGL((qkv_post_kernel<float, float>), grid, block, 0, st, sb, qkv, chunks,
                       chunk_stride, row_stride, col0, Hq, Hkv, hd, g.qk_norm, g.rms_eps,
                       (const float *)c->g_q, (const float *)c->g_k, c->rope_cos, c->rope_sin,
                       (float *)c->qrot, (float *)c->kbuf, (float *)c->vbuf, slot_elems, c->t_cap, 0);
  }
  return hipGetLastError();
}

}  // namespace dart
