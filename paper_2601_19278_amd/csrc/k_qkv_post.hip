// After the fused Q/K/V projection: per-head RMSNorm of q and k (optional), rotary
// positions, and the append of the new K/V rows to the draft layer's K/V buffers.
// The draft is a single layer (paper Sec. 3.2), so K/V of a row depend on that row only and
// can be kept across draft-verify iterations.
#include "common.h"
#include "dart_internal.h"

namespace dart {

// grid (pass rows, ceil((Hq + 2*Hkv) / 8)), block = 4 wavefronts, two heads each.  Lane l < hd/2
// holds elements l and l + hd/2 of a head, the two a rotary rotation mixes, so a head needs no
// LDS and no barrier; the head's sum of squares is a wavefront reduction.  The chunk partials
// of both heads are requested before either is used.
// Pass row i is position pos of sequence b (SeqBatch); q is produced for query rows only and
// stored at the compact index b*K + j; k and v of every row go to the sequence's K/V slot.
// T: storage type of the norm gains; CT: element type of q and of the K/V buffers.
constexpr int QKV_POST_WAVES = 4, QKV_POST_HPW = 2;
static_assert(QKV_POST_HPW == 2, "the early exit below names both heads");
template <typename T, typename CT>
__global__ __launch_bounds__(64 * QKV_POST_WAVES) void qkv_post_kernel(
    SeqBatch sb, const float *__restrict__ qkv, int chunks, size_t chunk_stride, int row_stride,
    int col0, int Hq, int Hkv, int hd, int qk_norm, float eps, const T *__restrict__ q_gain,
    const T *__restrict__ k_gain, const float *__restrict__ cos_tab,
    const float *__restrict__ sin_tab, CT *__restrict__ q_out, CT *__restrict__ kbuf,
    CT *__restrict__ vbuf, size_t slot_elems, int t_cap, int tiled) {
  const int i = blockIdx.x;
  const int h0 = (blockIdx.y * QKV_POST_WAVES + (threadIdx.x >> 6)) * QKV_POST_HPW;
  const int lane = threadIdx.x & 63, half = hd >> 1, heads = Hq + 2 * Hkv;
  if (h0 >= heads) return;                        // uniform per wavefront, like the skips below
  int b, pos, qi;
  seq_of_row(sb, i, b, pos, qi);
  const bool act = lane < half;
  kbuf += (size_t)sb.slot[b] * slot_elems;
  vbuf += (size_t)sb.slot[b] * slot_elems;
  const int t0 = lane, t1 = lane + half;          // the lane's two elements of a head
  // chunk partials: up to 8 chunks in flight per head, added in index order
  float x0[QKV_POST_HPW], x1[QKV_POST_HPW];
  bool live[QKV_POST_HPW];
#pragma unroll
  for (int j = 0; j < QKV_POST_HPW; ++j) {
    const int hh = h0 + j;
    // heads past the end, and q heads of rows that are not query rows, are skipped
    live[j] = hh < heads && !(hh < Hq && qi < 0);
    x0[j] = x1[j] = 0.f;
  }
  if (!live[0] && !live[QKV_POST_HPW - 1]) return;   // (two heads per wavefront)
  for (int c0 = 0; c0 < chunks; c0 += 8) {
    float p0[QKV_POST_HPW][8], p1[QKV_POST_HPW][8];
#pragma unroll
    for (int j = 0; j < QKV_POST_HPW; ++j) {
      const float *src = qkv + (size_t)i * row_stride + ((h0 + j) * hd - col0);   // q, then k, then v heads
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const bool in = live[j] && act && c0 + u < chunks;
        p0[j][u] = in ? src[(size_t)(c0 + u) * chunk_stride + t0] : 0.f;
        p1[j][u] = in ? src[(size_t)(c0 + u) * chunk_stride + t1] : 0.f;
      }
    }
#pragma unroll
    for (int j = 0; j < QKV_POST_HPW; ++j)
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (c0 + u < chunks) {
          x0[j] += p0[j][u];
          x1[j] += p1[j][u];
        }
  }
  const float c = act ? cos_tab[(size_t)pos * half + lane] : 0.f, s = act ? sin_tab[(size_t)pos * half + lane] : 0.f;

#pragma unroll
  for (int j = 0; j < QKV_POST_HPW; ++j) {
    if (!live[j]) continue;
    const int hh = h0 + j;
    const bool is_q = hh < Hq, is_k = !is_q && hh < Hq + Hkv;
    float a0 = x0[j], a1 = x1[j];
    if (!is_q && !is_k) {                         // value head: store as is
      const int g = hh - Hq - Hkv;
      if (act) {
        if (tiled) {
          vbuf[(size_t)g * hd * t_cap + attn_vt_index(pos, t0, hd)] = from_f32<CT>(a0);
          vbuf[(size_t)g * hd * t_cap + attn_vt_index(pos, t1, hd)] = from_f32<CT>(a1);
        } else {
          vbuf[((size_t)g * t_cap + pos) * hd + t0] = from_f32<CT>(a0);
          vbuf[((size_t)g * t_cap + pos) * hd + t1] = from_f32<CT>(a1);
        }
      }
      continue;
    }
    if (qk_norm) {
      const float ss = wave_sum_dpp(act ? a0 * a0 + a1 * a1 : 0.f);
      const float rinv = 1.0f / sqrtf(ss / (float)hd + eps);
      const T *gain = is_q ? q_gain : k_gain;
      if (act) {
        a0 = a0 * rinv * to_f32(gain[t0]);
        a1 = a1 * rinv * to_f32(gain[t1]);
      }
    }
    if (!act) continue;
    const float y0 = a0 * c - a1 * s, y1 = a1 * c + a0 * s;
    if (is_q) {
      CT *dst = q_out + ((size_t)(b * sb.K + qi) * Hq + hh) * hd;
      dst[t0] = from_f32<CT>(y0);
      dst[t1] = from_f32<CT>(y1);
    } else {
      const int g = hh - Hq;
      if (tiled) {
        kbuf[(size_t)g * hd * t_cap + attn_k_index(pos, t0, hd)] = from_f32<CT>(y0);
        kbuf[(size_t)g * hd * t_cap + attn_k_index(pos, t1, hd)] = from_f32<CT>(y1);
      } else {
        kbuf[((size_t)g * t_cap + pos) * hd + t0] = from_f32<CT>(y0);
        kbuf[((size_t)g * t_cap + pos) * hd + t1] = from_f32<CT>(y1);
      }
    }
  }
}

// K/V-only passes of many rows (the K/V build of a long prefix; fp16 operand-tile buffers): one
// workgroup per (sequence, aligned block of 32 keys, K/V head).  The per-row arithmetic is that
// of qkv_post_kernel, operation for operation (rows appended by either kernel share a buffer and
// must agree bit for bit); what differs is the store: the block's K and V rows are collected in
// LDS and written as whole 16-byte operand-tile pieces -- a K tile lane holds 8 dims of one key,
// a V^T tile lane holds 8 keys of one dim -- instead of one 2-byte store per element.  A block
// that the pass covers only partly keeps the other keys' stored values (K: lanes of keys outside
// the range do not store; V^T: the 16 bytes are read, merged and written back; no other
// workgroup of the launch touches them).
struct KvBlocks {
  int off[DART_SEQ_GROUP + 1];     // prefix sums of the sequences' 32-key blocks in this pass
};
constexpr int KVT_WAVES = 8, KVT_KEYS = 32;
template <typename T>
__global__ __launch_bounds__(64 * KVT_WAVES) void kv_post_tiles_kernel(
    SeqBatch sb, KvBlocks kb, const float *__restrict__ qkv, int chunks, size_t chunk_stride,
    int row_stride, int Hkv, int hd, int qk_norm, float eps, const T *__restrict__ k_gain,
    const float *__restrict__ cos_tab, const float *__restrict__ sin_tab, f16_t *__restrict__ kbuf,
    f16_t *__restrict__ vbuf, size_t slot_elems, int t_cap) {
  __shared__ __align__(16) f16_t ks[KVT_KEYS][128];
  __shared__ __align__(16) f16_t vs[KVT_KEYS][128];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, half = hd >> 1;
  const int g = blockIdx.y;
  int b = 0;
  while (b + 1 < sb.B && (int)blockIdx.x >= kb.off[b + 1]) ++b;
  const int p0 = sb.pos0[b], p1 = p0 + (sb.row_off[b + 1] - sb.row_off[b]);   // positions of the pass
  const int P = (p0 / KVT_KEYS + ((int)blockIdx.x - kb.off[b])) * KVT_KEYS;    // first key of the block
  const int lo = max(p0, P) - P, hi = min(p1, P + KVT_KEYS) - P;               // keys [lo, hi) are new
  const bool act = lane < half;
  const int t0 = lane, t1 = lane + half;

  // rows of the block, four per wavefront: chunk partials of the K head and of the V head
  for (int x = lo + wave; x < hi; x += KVT_WAVES) {
    const int pos = P + x, i = sb.row_off[b] + (pos - p0);
    const float *ksrc = qkv + (size_t)i * row_stride + g * hd;             // column 0 = first K column
    const float *vsrc = ksrc + Hkv * hd;
    float a0 = 0.f, a1 = 0.f, v0 = 0.f, v1 = 0.f;
    for (int c0 = 0; c0 < chunks; c0 += 8) {
      float pk0[8], pk1[8], pv0[8], pv1[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const bool in = act && c0 + u < chunks;
        const size_t o = (size_t)(c0 + u) * chunk_stride;
        pk0[u] = in ? ksrc[o + t0] : 0.f;
        pk1[u] = in ? ksrc[o + t1] : 0.f;
        pv0[u] = in ? vsrc[o + t0] : 0.f;
        pv1[u] = in ? vsrc[o + t1] : 0.f;
      }
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (c0 + u < chunks) {
          a0 += pk0[u];
          a1 += pk1[u];
          v0 += pv0[u];
          v1 += pv1[u];
        }
    }
    const float cs = act ? cos_tab[(size_t)pos * half + lane] : 0.f, sn = act ? sin_tab[(size_t)pos * half + lane] : 0.f;
    if (qk_norm) {
      const float ss = wave_sum_dpp(act ? a0 * a0 + a1 * a1 : 0.f);
      const float rinv = 1.0f / sqrtf(ss / (float)hd + eps);
      if (act) {
        a0 = a0 * rinv * to_f32(k_gain[t0]);
        a1 = a1 * rinv * to_f32(k_gain[t1]);
      }
    }
    if (act) {
      const float y0 = a0 * cs - a1 * sn, y1 = a1 * cs + a0 * sn;
      ks[x][t0] = from_f32<f16_t>(y0);
      ks[x][t1] = from_f32<f16_t>(y1);
      vs[x][t0] = from_f32<f16_t>(v0);
      vs[x][t1] = from_f32<f16_t>(v1);
    }
  }
  __syncthreads();

  const size_t head = (size_t)sb.slot[b] * slot_elems + (size_t)g * hd * t_cap +
                      (size_t)(P / ATTN_KEY_CHUNK) * ATTN_KEY_CHUNK * hd;    // this chunk of this head
  const int pc = P % ATTN_KEY_CHUNK;                                          // block's place in its chunk
  const int col = lane & 15, gq = lane >> 4;
  // K tiles: (key tile kt of the block, k-step ks2): lane = 8 dims of one key
  for (int tile = wave; tile < 2 * (hd / 32); tile += KVT_WAVES) {
    const int kt = tile / (hd / 32), ks2 = tile % (hd / 32);
    const int x = 16 * kt + col;
    if (x >= lo && x < hi) {
      const uint4 v = *reinterpret_cast<const uint4 *>(&ks[x][32 * ks2 + 8 * gq]);
      const size_t at = head + ((size_t)((pc / 16 + kt) * (hd / 32) + ks2) * 64 + lane) * 8;
      *reinterpret_cast<uint4 *>(kbuf + at) = v;
    }
  }
  // V^T tiles: (dim tile dt, this 32-key block): lane = 8 keys of one dim, keys 4 gq + e and
  // 16 + 4 gq + e (e < 4), the order attn_vt_position stores them in
  for (int dt = wave; dt < hd / 16; dt += KVT_WAVES) {
    const int dim = 16 * dt + col;
    const size_t at = head + ((size_t)(dt * (ATTN_KEY_CHUNK / 32) + pc / 32) * 64 + lane) * 8;
    union { uint4 u; f16_t e[8]; } w;
    const bool whole = lo == 0 && hi == KVT_KEYS;
    if (!whole) w.u = *reinterpret_cast<const uint4 *>(vbuf + at);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int x = (e < 4 ? 0 : 16) + 4 * gq + (e & 3);
      if (whole || (x >= lo && x < hi)) w.e[e] = vs[x][dim];
    }
    *reinterpret_cast<uint4 *>(vbuf + at) = w.u;
  }
}

hipError_t launch_qkv_post(const dart_ctx *c, const SeqBatch &sb, const float *qkv, int chunks,
                           size_t chunk_stride, int row_stride, int col0, hipStream_t st) {
  const dart_config &g = c->cfg;
  const int Hq = g.n_q_heads, Hkv = g.n_kv_heads, hd = g.head_dim;
  const size_t slot_elems = (size_t)Hkv * c->t_cap * hd;
  if (hd > 128 || (hd & 1)) return hipErrorInvalidValue;
  if (g.dtype == DART_BF16 && sb.K == 0 && col0 == Hq * hd && sb.row_off[sb.B] >= 64) {
    // a K/V-only pass of many rows: whole operand-tile pieces per store
    KvBlocks kb;
    kb.off[0] = 0;
    for (int b = 0; b < sb.B; ++b) {
      const int p0 = sb.pos0[b], p1 = p0 + (sb.row_off[b + 1] - sb.row_off[b]);
      kb.off[b + 1] = kb.off[b] + (p1 > p0 ? (p1 - 1) / KVT_KEYS - p0 / KVT_KEYS + 1 : 0);
    }
    hipLaunchKernelGGL(kv_post_tiles_kernel<bf16_t>, dim3(kb.off[sb.B], Hkv), dim3(64 * KVT_WAVES), 0, st,
                       sb, kb, qkv, chunks, chunk_stride, row_stride, Hkv, hd, g.qk_norm, g.rms_eps,
                       (const bf16_t *)c->g_k, c->rope_cos, c->rope_sin, (f16_t *)c->kbuf,
                       (f16_t *)c->vbuf, slot_elems, c->t_cap);
    return hipGetLastError();
  }
  constexpr int per_block = QKV_POST_WAVES * QKV_POST_HPW;
  dim3 grid(sb.row_off[sb.B], (Hq + 2 * Hkv + per_block - 1) / per_block), block(64 * QKV_POST_WAVES);
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
