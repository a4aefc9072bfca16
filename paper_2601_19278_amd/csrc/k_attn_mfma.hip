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
// is taken as (lane group, e) <-> key 16*(e/4) + 4*(l/16) + e%4.  V^T is stored with the keys
// of every 32-key block permuted by the same map (attn_vt_position), so that the matching A
// operand is 16 contiguous bytes, and probabilities never leave registers.
//
// Work split: one workgroup per (128-key split, K/V head, sequence).  The step is bound by
// memory latency, not bandwidth or arithmetic, so the whole K and V^T chunk of the split
// (64 KiB at head_dim 128) is requested at once: every wavefront issues its share of 1 KiB
// global -> LDS tile copies (no registers involved, tiles land in MFMA operand order) and the
// workgroup waits for them once.  Then wavefront w handles query tile(s) w, w+4 over the
// chunk's keys -- or, when there are fewer than 4 query tiles, a query tile over a part of
// the keys, written as a sub-split.  Split partials are merged by attn_merge_kernel.
#include "common.h"
#include "dart_internal.h"

namespace dart {

union F16x8 {
  f16x8_t v;
  uint4 u;
  f16_t e[8];
};

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((address_space(3))) void *lptr_t;

// One wavefront copies 1 KiB to LDS: lane l moves the 16 bytes at base + off to
// lds_base + 16*l.  lds_base is wave-uniform.  Completion is counted by vmcnt.
__device__ __forceinline__ void attn_copy_tile(uint32_t lds_base, uint32_t off, const void *base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_base), "v"(off), "s"(base)
               : "memory");
}

constexpr int ATTN_BLOCKS = ATTN_KEY_CHUNK / 32;   // 32-key blocks per split

// MTW: query tiles per wavefront (1 or 2).  NSUB: key sub-ranges a split is cut into when
// there are fewer query tiles than wavefronts (1, 2 or 4; NSUB * tiles <= 4).
template <int HD, int MTW, int NSUB>
__global__ __launch_bounds__(256) void attn_split_mfma_kernel(
    SeqBatch sb,
    const f16_t *__restrict__ q,      // [B*K][Hq][HD], query rows in compact order
    const f16_t *__restrict__ kbuf,   // [slot][Hkv][t_cap][HD]
    const f16_t *__restrict__ vtbuf,  // [slot][Hkv][HD][t_cap], keys permuted within 32-blocks
    size_t slot_elems, int t_cap, int tiles, int Hq, int group, float scale, int nsplit_total,
    float *__restrict__ o_part, float *__restrict__ ml_part) {
  constexpr int KS = HD / 32;        // k-steps of the score product
  constexpr int DT = HD / 16;        // output dim tiles
  constexpr int KT = ATTN_KEY_CHUNK / 16;
  __shared__ u32x4_t ktile[KT][KS][64];            // K operand tiles: 16 keys x 32 dims
  __shared__ u32x4_t vtile[DT][ATTN_BLOCKS][64];   // V^T operand tiles: 16 dims x 32 keys
  const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
  const int Kq = sb.K, n = sb.n[b];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int col = lane & 15, gq = lane >> 4;
  const int QV = Kq * group;
  const int T = n + Kq - 1;
  const int j0 = split * ATTN_KEY_CHUNK;
  if (j0 >= T) return;                                   // the merge never reads this split

  // request the whole chunk: tile copies are dealt round-robin to the wavefronts
  const f16_t *kb = kbuf + sb.slot[b] * slot_elems + (size_t)g * t_cap * HD + (size_t)j0 * HD;
  const f16_t *vt = vtbuf + sb.slot[b] * slot_elems + (size_t)g * HD * t_cap + j0;
  {
    constexpr int NK = KT * KS, NV = DT * ATTN_BLOCKS;
    // K tile (kt, ks): lane (gq, col) <- dims 32*ks + 8*gq.. of key 16*kt + col
    const uint32_t koff = (uint32_t)(col * HD + 8 * gq) * 2u;
#pragma unroll
    for (int i = 0; i < NK / 4; ++i) {
      const int t = wave + 4 * i, kt = t / KS, ks = t % KS;
      attn_copy_tile((uint32_t)(uintptr_t)(lptr_t)&ktile[kt][ks][0],
                     koff + (uint32_t)(16 * kt * HD + 32 * ks) * 2u, kb);
    }
    // V^T tile (dt, blk): lane (gq, col) <- stored positions 32*blk + 8*gq.. of dim 16*dt + col
    const uint32_t voff = (uint32_t)(col * t_cap + 8 * gq) * 2u;
#pragma unroll
    for (int i = 0; i < NV / 4; ++i) {
      const int t = wave + 4 * i, dt = t / ATTN_BLOCKS, blk = t % ATTN_BLOCKS;
      attn_copy_tile((uint32_t)(uintptr_t)(lptr_t)&vtile[dt][blk][0],
                     voff + (uint32_t)(16 * dt * t_cap + 32 * blk) * 2u, vt);
    }
  }

  // this wavefront's query tiles and key blocks
  const int sub = NSUB == 1 ? 0 : wave / (4 / NSUB);      // key sub-range
  const int a0 = NSUB == 1 ? wave : wave % (4 / NSUB);    // first query tile
  constexpr int BPS = ATTN_BLOCKS / NSUB;                 // key blocks per sub-range
  const bool active = a0 < tiles;

  // B operands of the score product: this lane's query column, all k-steps
  F16x8 qop[MTW][KS];
  int qrow[MTW];                     // query row i of this lane's column (-1: padding)
  size_t qslot[MTW];                 // global query-vector index
#pragma unroll
  for (int a = 0; a < MTW; ++a) {
    const int ql = 16 * (a0 + 4 * a) + col;
    const bool ok = active && ql < QV;
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

  f32x4_t acc[MTW][DT];
  float m[MTW], l[MTW];
#pragma unroll
  for (int a = 0; a < MTW; ++a) {
    m[a] = -3.0e38f;
    l[a] = 0.f;
#pragma unroll
    for (int t = 0; t < DT; ++t) acc[a][t] = {0.f, 0.f, 0.f, 0.f};
  }

  // every copy of every wavefront has landed once all have waited and met at the barrier
  asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");

  if (active) {
#pragma unroll
    for (int bi = 0; bi < BPS; ++bi) {
      const int blk = sub * BPS + bi;
      const int jb = j0 + 32 * blk;
      if (jb < T) {                                       // wave-uniform
        F16x8 kop[2][KS], vop[DT];
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
          for (int ks = 0; ks < KS; ++ks)
            kop[tt][ks].v = __builtin_bit_cast(f16x8_t, ktile[2 * blk + tt][ks][lane]);
#pragma unroll
        for (int t = 0; t < DT; ++t) vop[t].v = __builtin_bit_cast(f16x8_t, vtile[t][blk][lane]);

#pragma unroll
        for (int a = 0; a < MTW; ++a) {
          f32x4_t s[2];
#pragma unroll
          for (int tt = 0; tt < 2; ++tt) {
            s[tt] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
              s[tt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(kop[tt][ks].v, qop[a][ks].v, s[tt], 0, 0, 0);
          }
          // mask + running soft-max statistics of this lane's query column
          const int last = n - 1 + qrow[a];        // padding columns (qrow -1) see nothing
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
          for (int t = 0; t < DT; ++t) {
            acc[a][t] *= corr;
            acc[a][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(vop[t].v, pop.v, acc[a][t], 0, 0, 0);
          }
        }
      }
    }

#pragma unroll
    for (int a = 0; a < MTW; ++a) {
      if (qrow[a] < 0) continue;
      const size_t slot = qslot[a] * nsplit_total + (size_t)split * NSUB + sub;
#pragma unroll
      for (int t = 0; t < DT; ++t)
        *reinterpret_cast<float4 *>(o_part + slot * HD + 16 * t + 4 * gq) =
            make_float4(acc[a][t][0], acc[a][t][1], acc[a][t][2], acc[a][t][3]);
      if (gq == 0) {
        ml_part[slot * 2] = m[a];
        ml_part[slot * 2 + 1] = l[a];
      }
    }
  }
}

// Key sub-ranges per split for a given number of query tiles (see the kernel).
int attn_mfma_nsub(int Kq, int group) {
  const int tiles = (Kq * group + 15) / 16;
  return tiles == 1 ? 4 : (tiles == 2 ? 2 : 1);
}

template <int HD, int MTW, int NSUB>
static hipError_t launch_one(const dart_ctx *c, const SeqBatch &sb, int nsplit, int tiles,
                             hipStream_t st) {
  const dart_config &g = c->cfg;
  const size_t slot_elems = (size_t)g.n_kv_heads * c->t_cap * HD;
  hipLaunchKernelGGL((attn_split_mfma_kernel<HD, MTW, NSUB>), dim3(nsplit, g.n_kv_heads, sb.B),
                     dim3(256), 0, st, sb, (const f16_t *)c->qrot, (const f16_t *)c->kbuf,
                     (const f16_t *)c->vbuf, slot_elems, c->t_cap, tiles, g.n_q_heads,
                     g.n_q_heads / g.n_kv_heads, 1.0f / sqrtf((float)HD), nsplit * NSUB, c->att_part,
                     c->att_ml);
  return hipGetLastError();
}

// nsplit: 128-key splits of the longest sequence; the partial buffers hold
// nsplit * attn_mfma_nsub() entries per query vector.
hipError_t launch_attention_bf16(const dart_ctx *c, const SeqBatch &sb, int nsplit, hipStream_t st) {
  const dart_config &g = c->cfg;
  const int tiles = (sb.K * (g.n_q_heads / g.n_kv_heads) + 15) / 16;
  if (tiles > 8) return hipErrorInvalidValue;
  if (g.head_dim == 128) {
    if (tiles == 1) return launch_one<128, 1, 4>(c, sb, nsplit, tiles, st);
    if (tiles == 2) return launch_one<128, 1, 2>(c, sb, nsplit, tiles, st);
    if (tiles <= 4) return launch_one<128, 1, 1>(c, sb, nsplit, tiles, st);
    return launch_one<128, 2, 1>(c, sb, nsplit, tiles, st);
  }
  if (tiles == 1) return launch_one<64, 1, 4>(c, sb, nsplit, tiles, st);
  if (tiles == 2) return launch_one<64, 1, 2>(c, sb, nsplit, tiles, st);
  if (tiles <= 4) return launch_one<64, 1, 1>(c, sb, nsplit, tiles, st);
  return launch_one<64, 2, 1>(c, sb, nsplit, tiles, st);
}

}  // namespace dart
