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
//   S^T[key][q] = sum_dim K[key][dim] Q[q][dim]      A = K rows, B = Q
//   O^T[dim][q] = sum_key V^T[dim][key] P^T[key][q]   A = V^T rows (V is stored transposed)
// (both A operands are stored in the K/V buffers as the 1 KiB operand tiles themselves)
// The MFMA result layout (lane l: column l%16, rows 4*(l/16)+r) of S^T is, after the
// soft-max, directly the B operand of the second product if its 32-key contraction index
// is taken as (lane group, e) <-> key 16*(e/4) + 4*(l/16) + e%4.  V^T is stored with the keys
// of every 32-key block permuted by the same map (attn_vt_position), so that the matching A
// operand is 16 contiguous bytes, and probabilities never leave registers.
//
// Work split: the (sequence, K/V head, 128-key chunk) units of a launch form one list, cut into
// runs of `per` consecutive units, one workgroup per run; a run may end one (sequence, head) pair
// and begin the next, so ragged batches load every compute unit alike.  The step is bound by
// memory latency and bandwidth, not arithmetic, so a whole K and V^T chunk (64 KiB at head_dim
// 128) is requested at once: K and V^T are stored as the MFMA operand tiles themselves, every
// wavefront issues its share of 1 KiB global -> LDS tile copies (no registers involved) and the
// workgroup waits for them once.  With per > 1 the chunk buffer is doubled and the copies of the
// next unit are in flight while the current one is computed; the running (max, sum, output) of
// a query column is carried across the chunks of one pair, so one partial per (run, pair) is
// written instead of one per chunk.  With TW query-tile slots (1, 2, 4 or 8, at least the number
// of 16-column query tiles) a workgroup of NW wavefronts cuts every chunk's keys into NW / TW
// sub-ranges: wavefront w handles query tile w % TW over sub-range w / TW, and each sub-range is
// written as a partial of its own.  Partials are merged by attn_merge_kernel.
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
// lds_base + 16*l.  lds_base is wave-uniform.  Completion is counted by vmcnt.  The K/V stream
// is read once per call: non-temporal (measured 71 -> 67 us at 128 rows, neutral at 8).
__device__ __forceinline__ void attn_copy_tile(uint32_t lds_base, uint32_t off, const void *base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt"
               :
               : "s"(lds_base), "v"(off), "s"(base)
               : "memory");
}

constexpr int ATTN_BLOCKS = ATTN_KEY_CHUNK / 32;   // 32-key blocks per chunk

// NW: wavefronts per workgroup (4 or 8).  TW: query-tile slots (see above; NW / TW <= 4).
// Dynamic LDS: one chunk buffer (work.per == 1) or two.  Grid: ceil(units / work.per).
template <int HD, int NW, int TW>
__global__ __launch_bounds__(64 * NW) void attn_split_mfma_kernel(
    SeqBatch sb, AttnWork work,
    const f16_t *__restrict__ q,      // [B*K][Hq][HD], query rows in compact order
    const f16_t *__restrict__ kbuf,   // [slot][Hkv][chunk][K operand tiles]
    const f16_t *__restrict__ vtbuf,  // [slot][Hkv][chunk][V^T operand tiles]
    size_t slot_elems, int t_cap, int tiles, int Hq, int group, float scale, int nsplit_total,
    float *__restrict__ o_part, float *__restrict__ ml_part) {
  constexpr int KS = HD / 32;        // k-steps of the score product
  constexpr int DT = HD / 16;        // output dim tiles
  constexpr int KT = ATTN_KEY_CHUNK / 16;
  constexpr int NK = KT * KS;        // K operand tiles of a chunk: 16 keys x 32 dims each
  constexpr int NV = DT * ATTN_BLOCKS;   // V^T operand tiles: 16 dims x 32 keys each
  extern __shared__ u32x4_t attn_lds[];  // [buffer][NK + NV tiles][64 lanes]
  const int Hkv = Hq / group, Kq = sb.K, QV = Kq * group;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int col = lane & 15, gq = lane >> 4;
  const int u0 = blockIdx.x * work.per;
  const int u1 = min(u0 + work.per, work.cum[sb.B] * Hkv);

  // unit u -> (sequence b, head g, chunk); b only grows along a run
  int b = 0, g, chunk, cb;
  auto decode = [&](int u, int &b_, int &g_, int &chunk_, int &cb_) {
    while (b_ + 1 < sb.B && u >= work.cum[b_ + 1] * Hkv) ++b_;
    cb_ = work.cum[b_ + 1] - work.cum[b_];
    const int r = u - work.cum[b_] * Hkv;
    g_ = r / cb_;
    chunk_ = r - g_ * cb_;
  };
  // request a whole chunk into buffer buf: a tile copy moves 1 KiB of contiguous memory; the
  // copies are dealt round-robin to the wavefronts
  const uint32_t lds0 = (uint32_t)(uintptr_t)(lptr_t)attn_lds;
  const uint32_t loff = (uint32_t)lane * 16u;
  auto request = [&](int b_, int g_, int chunk_, int buf) {
    const size_t at = sb.slot[b_] * slot_elems + (size_t)g_ * t_cap * HD +
                      (size_t)chunk_ * ATTN_KEY_CHUNK * HD;
    const f16_t *kc = kbuf + at, *vc = vtbuf + at;
    const uint32_t base = lds0 + (uint32_t)buf * (NK + NV) * 1024u;
#pragma unroll
    for (int i = 0; i < NK / NW; ++i) {
      const int t = wave + NW * i;
      attn_copy_tile(base + (uint32_t)t * 1024u, loff + (uint32_t)t * 1024u, kc);
    }
#pragma unroll
    for (int i = 0; i < NV / NW; ++i) {
      const int t = wave + NW * i;
      attn_copy_tile(base + (uint32_t)(NK + t) * 1024u, loff + (uint32_t)t * 1024u, vc);
    }
  };
  decode(u0, b, g, chunk, cb);
  request(b, g, chunk, 0);

  // this wavefront's query tile and key blocks
  constexpr int NSUB = NW / TW, MTW = 1;
  const int sub = wave / TW;                              // key sub-range
  const int a0 = wave % TW;                               // query tile
  constexpr int BPS = ATTN_BLOCKS / NSUB;                 // key blocks per sub-range
  const bool active = a0 < tiles;

  F16x8 qop[MTW][KS];                // B operands of the score product: this lane's query column
  int qrow[MTW];                     // query row i of this lane's column (-1: padding)
  size_t qslot[MTW];                 // global query-vector index
  f32x4_t acc[MTW][DT];
  float m[MTW], l[MTW];
  bool fresh = true;                 // the next unit opens a (sequence, head) pair

  for (int u = u0; u < u1; ++u) {
    if (fresh) {
      fresh = false;
      u32x4_t qraw[MTW][KS];
#pragma unroll
      for (int a = 0; a < MTW; ++a) {
        const int ql = 16 * (a0 + TW * a) + col;
        const bool ok = active && ql < QV;
        const int i = ok ? ql / group : 0, hg = ok ? ql % group : 0;
        qrow[a] = ok ? i : -1;
        qslot[a] = (size_t)(b * Kq + i) * Hq + (size_t)g * group + hg;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          if (ok)
            qraw[a][ks] = *reinterpret_cast<const u32x4_t *>(q + qslot[a] * HD + 32 * ks + 8 * gq);
          else
            qraw[a][ks] = u32x4_t{0, 0, 0, 0};
        }
      }
      // The query loads are consumed here, inside the branch: the compiler's wait for them
      // would otherwise sit at their first use below, behind the next unit's request, and
      // drain that request (its copies are counted by the same counter) in every iteration.
#pragma unroll
      for (int a = 0; a < MTW; ++a) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          u32x4_t v = qraw[a][ks];
          asm volatile("" : "+v"(v));
          qop[a][ks].v = __builtin_bit_cast(f16x8_t, v);
        }
        m[a] = -3.0e38f;
        l[a] = 0.f;
#pragma unroll
        for (int t = 0; t < DT; ++t) acc[a][t] = {0.f, 0.f, 0.f, 0.f};
      }
    }
    // unit u has landed once every wavefront has waited for its own copies and all have met at
    // the barrier; passing it also means that every wavefront is done with unit u-1, whose
    // buffer the next request overwrites
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    int nb = b, ng = g, nchunk = chunk, ncb = cb;
    if (u + 1 < u1) {
      decode(u + 1, nb, ng, nchunk, ncb);
      request(nb, ng, nchunk, (u + 1 - u0) & 1);
    }
    const int n = sb.n[b];
    const int T = n + Kq - 1;
    if (active) {
      const u32x4_t *ktile = attn_lds + (size_t)((u - u0) & 1) * (NK + NV) * 64;
      const u32x4_t *vtile = ktile + NK * 64;
      const int j0 = chunk * ATTN_KEY_CHUNK;
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
              kop[tt][ks].v = __builtin_bit_cast(f16x8_t, ktile[((2 * blk + tt) * KS + ks) * 64 + lane]);
#pragma unroll
          for (int t = 0; t < DT; ++t)
            vop[t].v = __builtin_bit_cast(f16x8_t, vtile[(t * ATTN_BLOCKS + blk) * 64 + lane]);

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
            mloc = quad16_max(mloc);
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
            lsum = quad16_sum(lsum);
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
    }
    if (chunk == cb - 1 || u + 1 == u1) {
      // The pair ends here, or the run does: one partial per query column, numbered by the run
      // within the pair.  The NSUB wavefronts that hold the key sub-ranges of a query tile
      // first merge their (max, sum, output) through the chunk buffer that has just been
      // consumed (the next unit's copies go to the other one): half or a quarter of the bytes
      // to store here and to read back in the merge kernel.  The condition is uniform over the
      // workgroup, so the barriers are too; they order LDS traffic only.
      if constexpr (NSUB > 1) {
        constexpr int F = 4 * DT + 2;                              // floats per lane
        static_assert(MTW == 1 && TW * F * 256 <= (NK + NV) * 1024, "fits one chunk buffer");
        float *xb = reinterpret_cast<float *>(attn_lds + (size_t)((u - u0) & 1) * (NK + NV) * 64) +
                    (size_t)a0 * F * 64 + lane;
        // one sub-range at a time hands its state to the wavefront of sub-range 0
#pragma unroll
        for (int s2 = 1; s2 < NSUB; ++s2) {
          // everyone is done with the chunk (first round) / the previous hand-over has been read
          asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
          if (active && sub == s2) {
#pragma unroll
            for (int t = 0; t < DT; ++t)
#pragma unroll
              for (int r = 0; r < 4; ++r) xb[(4 * t + r) * 64] = acc[0][t][r];
            xb[(4 * DT) * 64] = m[0];
            xb[(4 * DT + 1) * 64] = l[0];
          }
          asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
          if (active && sub == 0) {
            const float m2 = xb[(4 * DT) * 64], l2 = xb[(4 * DT + 1) * 64];
            const float mn = fmaxf(m[0], m2);
            const float c0 = __expf(m[0] - mn), c1 = __expf(m2 - mn);
            l[0] = l[0] * c0 + l2 * c1;
            m[0] = mn;
#pragma unroll
            for (int t = 0; t < DT; ++t)
#pragma unroll
              for (int r = 0; r < 4; ++r) acc[0][t][r] = acc[0][t][r] * c0 + xb[(4 * t + r) * 64] * c1;
          }
        }
      }
      if (active && sub == 0) {
        const int pair0 = work.cum[b] * Hkv + g * cb;      // first unit of the pair
        const int seg = (int)blockIdx.x - pair0 / work.per;
#pragma unroll
        for (int a = 0; a < MTW; ++a) {
          if (qrow[a] < 0) continue;
          const size_t slot = qslot[a] * nsplit_total + (size_t)seg;
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
      fresh = true;
    }
    b = nb, g = ng, chunk = nchunk, cb = ncb;
  }
}

template <int HD, int NW, int TW>
static hipError_t launch_one(const dart_ctx *c, const SeqBatch &sb, const AttnWork &work, int nseg,
                             int tiles, hipStream_t st) {
  const dart_config &g = c->cfg;
  const size_t slot_elems = (size_t)g.n_kv_heads * c->t_cap * HD;
  auto kern = attn_split_mfma_kernel<HD, NW, TW>;
  const size_t chunk_bytes = (size_t)2 * ATTN_KEY_CHUNK * HD * sizeof(f16_t);   // K and V^T
  const size_t lds = chunk_bytes * (work.per > 1 ? 2 : 1);
  hipError_t e = raise_dynamic_lds_once(reinterpret_cast<const void *>(kern), (int)(2 * chunk_bytes));
  if (e != hipSuccess) return e;
  const int units = work.cum[sb.B] * g.n_kv_heads;
  hipLaunchKernelGGL(kern, dim3((units + work.per - 1) / work.per), dim3(64 * NW), lds, st, sb, work,
                     (const f16_t *)c->qrot, (const f16_t *)c->kbuf, (const f16_t *)c->vbuf,
                     slot_elems, c->t_cap, tiles, g.n_q_heads, g.n_q_heads / g.n_kv_heads,
                     1.0f / sqrtf((float)HD), nseg, c->att_part, c->att_ml);
  return hipGetLastError();
}

// work: the launch's unit list; nseg: partial slots per query vector.
hipError_t launch_attention_bf16(const dart_ctx *c, const SeqBatch &sb, const AttnWork &work,
                                 int nseg, hipStream_t st) {
  const dart_config &g = c->cfg;
  const int tiles = (sb.K * (g.n_q_heads / g.n_kv_heads) + 15) / 16;
  if (tiles > 8) return hipErrorInvalidValue;
  if (g.head_dim == 128) {
    if (tiles == 1) return launch_one<128, 4, 1>(c, sb, work, nseg, tiles, st);
    if (tiles == 2) return launch_one<128, 4, 2>(c, sb, work, nseg, tiles, st);
    if (tiles <= 4) return launch_one<128, 8, 4>(c, sb, work, nseg, tiles, st);
    return launch_one<128, 8, 8>(c, sb, work, nseg, tiles, st);
  }
  if (tiles == 1) return launch_one<64, 4, 1>(c, sb, work, nseg, tiles, st);
  if (tiles == 2) return launch_one<64, 4, 2>(c, sb, work, nseg, tiles, st);
  if (tiles <= 4) return launch_one<64, 8, 4>(c, sb, work, nseg, tiles, st);
  return launch_one<64, 8, 8>(c, sb, work, nseg, tiles, st);
}

}  // namespace dart
