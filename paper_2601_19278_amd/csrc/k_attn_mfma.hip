// Masked-position attention of the draft layer for the bf16 configuration, MFMA 16x16x32.
//
// q, the K/V buffers and the soft-max probabilities are held in fp16 (fp32 accumulate): they
// are the library's own intermediates, cost the same bytes as bf16, and their 11-bit
// significand keeps the rounding of the attention path an order of magnitude below the
// logit tolerance, which bf16's 8 bits do not (mask rows carry a tiny residual, so the
// final RMSNorm amplifies relative errors of the attention output).  Values are bounded
// (soft-max weights, normalised/rotated q and k); stores saturate at the fp16 maximum.
//
// K = up to 16 query rows times Hq/Hkv query heads share each K/V head, so the scores of
// one K/V head are a (keys x 128 dims) x (128 dims x up-to-128 queries) contraction: small,
// but a real dense one, and the K/V stream (read once) is what bounds it.
//
// The product is formed transposed so that a lane owns one query column throughout:
//   S^T[key][q] = sum_dim K[key][dim] Q[q][dim]      A = K rows (row-major buffer), B = Q
//   O^T[dim][q] = sum_key V^T[dim][key] P^T[key][q]   A = V^T rows (V is stored transposed)
// The MFMA result layout (lane l: column l%16, rows 4*(l/16)+r) of S^T is, after the
// soft-max, directly the B operand of the second product if its 32-key contraction index
// is taken as (lane group, e) <-> key 16*(e/4) + 4*(l/16) + e%4 -- V^T is loaded with the
// same index map, so probabilities never leave registers.
//
// Work split: grid (key split, K/V head, sequence x query-tile group), 4 wavefronts per workgroup.
// Every wavefront walks all keys of the split and computes the (cheap) scores and soft-max
// statistics redundantly; wavefront w accumulates only output dims [HD/4*w, HD/4*(w+1)).
// No LDS, no cross-wave merge; split partials are merged by attn_merge_kernel.
#include "common.h"
#include "dart_internal.h"

namespace dart {

union F16x8 {
  f16x8_t v;
  uint4 u;
  uint2 h[2];
  f16_t e[8];
};

template <int HD, int MT>
__global__ __launch_bounds__(256) void attn_split_mfma_kernel(
    SeqBatch sb,
    const f16_t *__restrict__ q,      // [B*K][Hq][HD], query rows in compact order
    const f16_t *__restrict__ kbuf,   // [slot][Hkv][t_cap][HD]
    const f16_t *__restrict__ vtbuf,  // [slot][Hkv][HD][t_cap]
    size_t slot_elems, int t_cap, int zgroups, int Hq, int group, int chunk, float scale,
    int nsplit, float *__restrict__ o_part, float *__restrict__ ml_part) {
  constexpr int KS = HD / 32;        // k-steps of the score product
  constexpr int DTW = HD / 64;       // output dim tiles per wavefront
  const int split = blockIdx.x, g = blockIdx.y;
  const int b = blockIdx.z / zgroups, a0 = (blockIdx.z % zgroups) * MT;
  const int Kq = sb.K, n = sb.n[b];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 15, gq = lane >> 4;
  const int QV = Kq * group;
  const int T = n + Kq - 1;
  const int j_begin = split * chunk;
  if (j_begin >= T) return;                              // the merge never reads this split
  const int j_end = min(j_begin + chunk, T);

  // B operands of the score product: this lane's query column, all k-steps, MT tiles
  F16x8 qop[MT][KS];
  int qrow[MT];                      // query row i of this lane's column (-1: padding)
  size_t qslot[MT];                  // global query-vector index
#pragma unroll
  for (int a = 0; a < MT; ++a) {
    const int ql = 16 * (a0 + a) + col;
    const bool ok = ql < QV;
    const int i = ok ? ql / group : 0, hg = ok ? ql % group : 0;
    qrow[a] = ok ? i : -1;
    qslot[a] = (size_t)(b * Kq + i) * Hq + (size_t)g * group + hg;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      if (ok)
        qop[a][ks].u = *reinterpret_cast<const uint4 *>(q + qslot[a] * HD + 32 * ks + 8 * gq);
      else
        qop[a][ks].u = make_uint4(0, 0, 0, 0);
    }
  }

  f32x4_t acc[MT][DTW];
  float m[MT], l[MT];
#pragma unroll
  for (int a = 0; a < MT; ++a) {
    m[a] = -3.0e38f;
    l[a] = 0.f;
#pragma unroll
    for (int t = 0; t < DTW; ++t) acc[a][t] = {0.f, 0.f, 0.f, 0.f};
  }

  const f16_t *kb = kbuf + sb.slot[b] * slot_elems + (size_t)g * t_cap * HD;
  const f16_t *vt = vtbuf + sb.slot[b] * slot_elems + (size_t)g * HD * t_cap;

  // A operands of one 32-key block: two 16-key tiles of K, and this wavefront's V^T dim tiles
  struct Block {
    F16x8 kop[2][KS], vop[DTW];
  };
  auto load_block = [&](int jb, Block &blk) {
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        blk.kop[tt][ks].u = *reinterpret_cast<const uint4 *>(
            kb + (size_t)(jb + 16 * tt + col) * HD + 32 * ks + 8 * gq);
#pragma unroll
    for (int t = 0; t < DTW; ++t) {
      const f16_t *row = vt + (size_t)(16 * (DTW * wave + t) + col) * t_cap + jb + 4 * gq;
      blk.vop[t].h[0] = *reinterpret_cast<const uint2 *>(row);
      blk.vop[t].h[1] = *reinterpret_cast<const uint2 *>(row + 16);
    }
  };

  Block nxt;
  if (j_begin < j_end) load_block(j_begin, nxt);
  for (int jb = j_begin; jb < j_end; jb += 32) {
    // software pipeline: the next block's K/V are in flight while this block is computed
    const Block cur = nxt;
    if (jb + 32 < j_end) load_block(jb + 32, nxt);
    const F16x8 (&kop)[2][KS] = cur.kop;
    const F16x8 (&vop)[DTW] = cur.vop;

#pragma unroll
    for (int a = 0; a < MT; ++a) {
      f32x4_t s[2];
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        s[tt] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          s[tt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(kop[tt][ks].v, qop[a][ks].v, s[tt], 0, 0, 0);
      }
      // mask + running soft-max statistics of this lane's query column
      const int last = n - 1 + qrow[a];            // qrow = -1 -> nothing visible beyond n-2; unused
      float mloc = -3.0e38f;
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int jk = jb + 16 * tt + 4 * gq + r;
          const bool vis = (qrow[a] >= 0) && (jk <= last);
          s[tt][r] = vis ? s[tt][r] * scale : -3.0e38f;
          mloc = fmaxf(mloc, s[tt][r]);
        }
      mloc = fmaxf(mloc, __shfl_xor(mloc, 16, DART_WAVE));
      mloc = fmaxf(mloc, __shfl_xor(mloc, 32, DART_WAVE));
      const float mn = fmaxf(m[a], mloc);
      const float corr = __expf(m[a] - mn);
      float lsum = 0.f;
      F16x8 pop;
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float p = s[tt][r] > -1.0e38f ? __expf(s[tt][r] - mn) : 0.f;
          lsum += p;
          pop.e[4 * tt + r] = (f16_t)p;
        }
      lsum += __shfl_xor(lsum, 16, DART_WAVE);
      lsum += __shfl_xor(lsum, 32, DART_WAVE);
      l[a] = l[a] * corr + lsum;
      m[a] = mn;
#pragma unroll
      for (int t = 0; t < DTW; ++t) {
        acc[a][t] *= corr;
        acc[a][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(vop[t].v, pop.v, acc[a][t], 0, 0, 0);
      }
    }
  }

#pragma unroll
  for (int a = 0; a < MT; ++a) {
    if (qrow[a] < 0) continue;
    const size_t slot = qslot[a] * nsplit + split;
#pragma unroll
    for (int t = 0; t < DTW; ++t) {
      const int dim = 16 * (DTW * wave + t) + 4 * gq;
      *reinterpret_cast<float4 *>(o_part + slot * HD + dim) =
          make_float4(acc[a][t][0], acc[a][t][1], acc[a][t][2], acc[a][t][3]);
    }
    if (wave == 0 && gq == 0) {
      ml_part[slot * 2] = m[a];
      ml_part[slot * 2 + 1] = l[a];
    }
  }
}

template <int HD, int MT>
static hipError_t launch_one(const dart_ctx *c, const SeqBatch &sb, int chunk, int nsplit,
                             int zgroups, hipStream_t st) {
  const dart_config &g = c->cfg;
  const size_t slot_elems = (size_t)g.n_kv_heads * c->t_cap * HD;
  hipLaunchKernelGGL((attn_split_mfma_kernel<HD, MT>),
                     dim3(nsplit, g.n_kv_heads, zgroups * sb.B), dim3(256), 0, st, sb,
                     (const f16_t *)c->qrot, (const f16_t *)c->kbuf, (const f16_t *)c->vbuf,
                     slot_elems, c->t_cap, zgroups, g.n_q_heads, g.n_q_heads / g.n_kv_heads, chunk,
                     1.0f / sqrtf((float)HD), nsplit, c->att_part, c->att_ml);
  return hipGetLastError();
}

int g_attn_mt = 3;        // query tiles per workgroup (tunable)

hipError_t launch_attention_bf16(const dart_ctx *c, const SeqBatch &sb, int chunk, int nsplit,
                                 hipStream_t st) {
  const dart_config &g = c->cfg;
  const int QV = sb.K * (g.n_q_heads / g.n_kv_heads);
  const int tiles = (QV + 15) / 16;
  const int MT = tiles >= g_attn_mt ? g_attn_mt : tiles;   // query tiles per workgroup
  const int zgroups = (tiles + MT - 1) / MT;
  if (g.head_dim == 128) {
    if (MT == 1) return launch_one<128, 1>(c, sb, chunk, nsplit, zgroups, st);
    if (MT == 2) return launch_one<128, 2>(c, sb, chunk, nsplit, zgroups, st);
    return launch_one<128, 3>(c, sb, chunk, nsplit, zgroups, st);
  }
  if (MT == 1) return launch_one<64, 1>(c, sb, chunk, nsplit, zgroups, st);
  if (MT == 2) return launch_one<64, 2>(c, sb, chunk, nsplit, zgroups, st);
  return launch_one<64, 3>(c, sb, chunk, nsplit, zgroups, st);
}

}  // namespace dart
