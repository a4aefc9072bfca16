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
// right after the MFMAs that free each register (several KiB in flight per wavefront).  Per
// strip the 8 partial 16x16 tiles are summed through LDS in a fixed order
// (deterministic), one barrier per strip.  When the k range is too long for the register
// budget the range is cut into chunks handled by different workgroups, and the consumer
// adds the chunk partials (also in fixed order).
#include <cstdio>

#include "common.h"
#include "dart_internal.h"
#include "topk_select.h"

namespace dart {

constexpr int GEMV_WAVES = 8;
constexpr int GEMV_THREADS = GEMV_WAVES * 64;
constexpr int GEMV_KPW_MAX = 20;          // k-steps (of 32 inputs) per wavefront per chunk

int gemv_bf16_chunks(int Kd) {
  const int KT = Kd / 32;
  return (KT + GEMV_WAVES * GEMV_KPW_MAX - 1) / (GEMV_WAVES * GEMV_KPW_MAX);
}

// Tunables (fixed after measurement; variables only in a -DDART_TUNING build).
DART_TUNABLE int g_gemv_wgs = 184;      // resident workgroups.  Fewer than the 256 compute units on purpose: measured on
                           // MI355X the weight stream peaks at 176-192 workgroups (LM head 6.6 TB/s against
                           // 6.2 TB/s with one per compute unit; 160 and fewer fall off again)
DART_TUNABLE int g_gemv_wgs_split = 224;  // the same for matrices whose k range is cut into chunks (QKV, O, MLP): best at 216-232
DART_TUNABLE int g_gemv_xcd = 2;        // strip-to-XCD assignment, see the kernel
DART_TUNABLE int g_gemv_depth = 0;      // 0 = default rolling-buffer depth for the k-slice length
DART_TUNABLE int g_gemv_nt = 1;         // weight tiles are read once: load them with the non-temporal hint
DART_TUNABLE int g_gemv_nt_min_mb = 100;  // ... for matrices (strip ranges) of at least this many MiB: smaller ones
                             // (QKV, O) partly survive in the last-level cache from step to step (measured -3 us)

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

template <bool NT>
__device__ __forceinline__ u32x4_t load_tile(const u32x4_t *p) {
  if constexpr (NT) {
    return __builtin_nontemporal_load(p);
  } else {
    return *p;
  }
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every
// outstanding global load (vmcnt(0)), which would drain the weight prefetch pipeline once
// per strip; the partial tiles exchanged here live in LDS, so waiting for LDS is enough.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// MT = 0: at most 8 activation rows.  The 16 B-operand columns then carry the hi parts of rows
// 0..7 in columns 0..7 and their lo parts in columns 8..15, so one MFMA per weight tile yields
// both products; result[m] = D[.][m] + D[.][m+8].
// MT >= 1: up to 16*MT rows as MT column tiles, separate hi and lo operands, 2*MT MFMAs per
// weight tile (MT = 1 is the 9..16-row case of the draft step; MT = 2, 4 serve the bulk K/V
// build of a long prefix, where each workgroup takes one block of 16*MT rows, blockIdx.y).
// All variants accumulate a row's hi products and lo products in two chains in k order and
// add the eight k-slice partials in the same order, so a row's result does not depend on the
// variant, on the number of rows, or on which call computed it.
// EXACT = true: every wavefront owns exactly KPW k-steps (the k range divides evenly), and
// the main loop is branch-free straight-line code -- the compiler can then keep D loads in
// flight with exact wait counts.  EXACT = false handles ragged k ranges (unusual shapes) with
// per-step guards and is not tuned.
// TK = true (the LM head with at most 8 rows, one k-chunk): the workgroup also keeps the logits of
// its strips in LDS and, after its last strip, selects per row the k best of them and their
// (max, sum exp) -- the per-position candidate extraction of Alg. 1 done where the logits are
// produced, so that no kernel has to read the vocabulary-wide rows again.  One wavefront per row;
// the row merge (topk_merge_kernel) then combines the workgroups' lists exactly as it combines
// the chunk lists of topk_kernel.  out may be null (logits not wanted).
constexpr int GEMV_TK_STRIPS = 64;        // strips of one workgroup whose logits fit its LDS buffer
template <int KPW, int D, int MT, bool NT, bool EXACT, bool TK = false>
__global__ __launch_bounds__(GEMV_THREADS) void gemv_bf16_kernel(
    const u32x4_t *__restrict__ Wp, // packed tiles, 64 x 16 bytes per tile
    const float *__restrict__ X,    // [M][Kd]
    int M, int KT, int kpw, int nchunks, int strip0, int nstrips, int n_cols,
    float *__restrict__ out, int out_stride, size_t chunk_stride, int xcd_map, GemvTopk tk) {
  static_assert(KPW % D == 0, "a register of the rolling buffer must serve the same slots in every strip");
  constexpr bool M8 = MT == 0;
  constexpr int NMT = M8 ? 1 : MT;                     // column tiles
  constexpr int NACC = M8 ? 1 : 2 * MT;                // accumulator tiles per strip
  constexpr int NBUF = NACC <= 2 ? 2 : 1;              // LDS double buffering while it fits
  __shared__ float part[NBUF][GEMV_WAVES][NACC * 256];
  __shared__ float wl[TK ? GEMV_TK_STRIPS : 1][128];   // TK: logits of this workgroup's strips, [row][16]
  static_assert(!TK || (MT == 0 && NBUF == 2), "candidate selection: at most 8 rows");
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 15, gq = lane >> 4;
  const int chunk = blockIdx.x % nchunks;
  const int nwg = gridDim.x / nchunks;
  int wg = blockIdx.x / nchunks;
  // Strip assignment.  Workgroups are dealt to the 8 XCDs round-robin (block i runs on XCD
  // i % 8, each with its own L2 and its own path to memory); block = wg * nchunks + chunk, so
  // the workgroups of one k-chunk fall into ncls = 8 / gcd(8, nchunks) classes (wg % ncls)
  // that share an XCD.  xcd_map 2: every class owns a contiguous 1/ncls of the strips and its
  // workgroups stride through it; 1: the workgroups of a class take adjacent strips of every
  // round; 0: strips dealt in launch order.  Measured on the LM head (184 workgroups, one
  // chunk): 235 / 228 / 227 us for modes 0 / 1 / 2.
  int s_step = nwg, s_end = nstrips;
  const int ncls = (nchunks & 1) ? 8 : ((nchunks & 2) ? 4 : ((nchunks & 4) ? 2 : 1));
  if (xcd_map == 1 && nwg % ncls == 0) wg = (wg % ncls) * (nwg / ncls) + wg / ncls;
  if (xcd_map == 2 && nwg % ncls == 0) {
    const int per_x = (nstrips + ncls - 1) / ncls, x = wg % ncls;
    s_step = nwg / ncls;
    s_end = min(nstrips, (x + 1) * per_x);
    wg = x * per_x + wg / ncls;
  }
  const int ks0 = (chunk * GEMV_WAVES + wave) * kpw;
  const int nk = EXACT ? KPW : max(0, min(kpw, KT - ks0));   // wave-uniform
  const int Kd = KT * 32;
  const int row_base = blockIdx.y * 16 * NMT;          // this workgroup's block of rows
  X += (size_t)row_base * Kd;
  out += (size_t)row_base * out_stride;
  M = min(M - row_base, 16 * NMT);

  // Rolling buffer of D weight tiles: register t % D serves slot t of every strip; the load
  // for its next slot is issued right after the MFMAs that free it, so about D KiB stay in
  // flight per wavefront across strip boundaries.  After the last strip the refills re-read
  // tiles of that same strip (in bounds, never used) so that the loop body has no branch.
  // The first D loads go out before the activations are fetched and converted, so the weight
  // stream is already running during that set-up.
  u32x4_t aop[D];
  int s = wg;                                          // strip index relative to strip0
  if (s < s_end) {
    const u32x4_t *tile = Wp + ((size_t)(strip0 + s) * KT + ks0) * 64 + lane;
#pragma unroll
    for (int r = 0; r < D; ++r)
      if (r < nk) aop[r] = load_tile<NT>(tile + (size_t)r * 64);
  }
  // B operands: activations of this wavefront's k slice, split into bf16 hi + bf16 lo
  // (x ~= hi + lo to ~2^-17) so that activations keep fp32-like accuracy while the weights
  // stay the exact bf16 values.
  bf16x8_t bop[NACC][KPW];
#pragma unroll
  for (int mt = 0; mt < NMT; ++mt) {
    const int xrow = M8 ? (col & 7) : 16 * mt + col;
#pragma unroll
    for (int t = 0; t < KPW; ++t) {
      union { bf16x8_t v; bf16_t e[8]; } h, l;
#pragma unroll
      for (int e = 0; e < 8; ++e) h.e[e] = l.e[e] = 0;
      if (t < nk && xrow < M) {
        const float *src = X + (size_t)xrow * Kd + (size_t)(ks0 + t) * 32 + 8 * gq;
        const float4 lo4 = *reinterpret_cast<const float4 *>(src);
        const float4 hi4 = *reinterpret_cast<const float4 *>(src + 4);
        const float x[8] = {lo4.x, lo4.y, lo4.z, lo4.w, hi4.x, hi4.y, hi4.z, hi4.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          h.e[e] = f32_to_bf16(x[e]);
          l.e[e] = f32_to_bf16(x[e] - bf16_to_f32(h.e[e]));
        }
      }
      if (M8) {
        bop[0][t] = col < 8 ? h.v : l.v;
      } else {
        bop[2 * mt][t] = h.v;
        bop[NACC > 1 ? 2 * mt + 1 : 0][t] = l.v;
      }
    }
  }

  int buf = 0;
  const int s_first = s;
  int n_done = 0;                                      // strips this workgroup has finished
  for (; s < s_end; s += s_step) {
    const int sn = s + s_step;
    const u32x4_t *cur = Wp + ((size_t)(strip0 + s) * KT + ks0) * 64 + lane;
    const u32x4_t *next = Wp + ((size_t)(strip0 + (sn < s_end ? sn : s)) * KT + ks0) * 64 + lane;
    f32x4_t acc[NACC];
#pragma unroll
    for (int i = 0; i < NACC; ++i) acc[i] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < KPW; ++t) {
      if (EXACT || t < nk) {
        const bf16x8_t a = __builtin_bit_cast(bf16x8_t, aop[t % D]);
#pragma unroll
        for (int i = 0; i < NACC; ++i)
          acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bop[i][t], acc[i], 0, 0, 0);
        if (EXACT) {
          aop[t % D] = load_tile<NT>(t + D < KPW ? cur + (size_t)(t + D) * 64
                                                   : next + (size_t)(t + D - KPW) * 64);
          // keep "MFMA, then the refill of its register" in program order: without this the
          // scheduler groups all MFMAs before all loads and the load queue drains each strip
          __builtin_amdgcn_sched_barrier(0);
        } else if (t + D < nk) {
          aop[t % D] = load_tile<NT>(cur + (size_t)(t + D) * 64);
        } else if ((t % D) < nk) {
          aop[t % D] = load_tile<NT>(next + (size_t)(t % D) * 64);
        }
      }
    }
    if (NBUF == 1) lds_barrier();                      // the previous strip's readers are done
#pragma unroll
    for (int i = 0; i < NACC; ++i)
      *reinterpret_cast<float4 *>(&part[buf][wave][i * 256 + lane * 4]) =
          make_float4(acc[i][0], acc[i][1], acc[i][2], acc[i][3]);
    lds_barrier();
    // D[row][c] of a tile lives in lane (row/4)*16 + c, register row%4.  MT = 0: lo products
    // sit in column m + 8 of the same tile; otherwise in the tile after the hi tile.
    for (int o = threadIdx.x; o < (M8 ? 128 : 256 * NMT); o += GEMV_THREADS) {
      const int mt = o >> 8, m = (o >> 4) & 15, row = o & 15;
      const int idx = (M8 ? 0 : 2 * mt * 256) + (((row >> 2) * 16) + m) * 4 + (row & 3);
      const int idx_lo = M8 ? idx + 32 : idx + 256;
      float v_hi = 0.f, v_lo = 0.f;
#pragma unroll
      for (int w = 0; w < GEMV_WAVES; ++w) v_hi += part[buf][w][idx];
#pragma unroll
      for (int w = 0; w < GEMV_WAVES; ++w) v_lo += part[buf][w][idx_lo];
      const int c = s * 16 + row, mm = 16 * mt + m;
      if constexpr (TK) {
        const bool real = mm < M && c < n_cols;
        wl[n_done][o] = real ? v_hi + v_lo : -3.0e38f;        // o = m * 16 + row
        if (real && out) out[(size_t)mm * out_stride + c] = v_hi + v_lo;
      } else {
        if (mm < M && c < n_cols)
          out[chunk * chunk_stride + (size_t)mm * out_stride + c] = v_hi + v_lo;
      }
    }
    if (NBUF == 2) buf ^= 1;
    ++n_done;
  }
  if constexpr (TK) {
    // Candidates of this workgroup: wavefront m takes row m over the n_done * 16 logits in LDS.
    __syncthreads();
    const int m = wave;
    if (m >= M) return;
    constexpr int NE = GEMV_TK_STRIPS * 16 / 64;         // entries per lane
    const int total = n_done * 16;
    const int ne = lane < total ? min(NE, (total - lane + 63) >> 6) : 0;
    float val[NE];
    float mx = -3.0e38f;
#pragma unroll
    for (int e = 0; e < NE; ++e) {
      const int i = lane + 64 * e;
      val[e] = e < ne ? wl[i >> 4][m * 16 + (i & 15)] : -3.0e38f;
      mx = fmaxf(mx, val[e]);
    }
    mx = wave_max_dpp(mx);
    float se = 0.f;
    uint32_t v[NE];
#pragma unroll
    for (int e = 0; e < NE; ++e) {
      // entries beyond the vocabulary (the padding outputs of the last strip) hold -3e38: they add
      // exp(-inf) = 0 and sort below every real logit; their keys are dropped below
      if (e < ne && val[e] > -1.0e38f) se += __expf(val[e] - mx);
      v[e] = val[e] > -1.0e38f ? f32_sortable(val[e]) : 0u;
    }
    se = wave_sum_dpp(se);
    const size_t slot = (size_t)m * gridDim.x + blockIdx.x;
    if (lane == 0) {
      tk.ms[slot * 2] = mx;
      tk.ms[slot * 2 + 1] = se;
    }
    // vocabulary index of the lane's e-th entry: strip s_first + (i / 16) * s_step, output i % 16
    uint64_t *sel = reinterpret_cast<uint64_t *>(&part[0][0][0]) + (size_t)wave * TOPK_CAP;
    static_assert(sizeof(part) >= GEMV_WAVES * TOPK_CAP * sizeof(uint64_t), "selection buffers fit");
    wave_select_indexed(
        v, ne, [&](int e) { const int i = lane + 64 * e; return (strip0 + s_first + (i >> 4) * s_step) * 16 + (i & 15); },
        tk.k, sel, [&](int r, uint64_t best) {
          tk.cand[slot * DART_MAX_TOPK + r] = (best >> 32) ? best : 0;   // value word 0 = a padding entry
        });
  }
}

template <int KPW, int D, bool EXACT>
static void gemv_launch(bool nt, int mt, const GemvTopk *tk, dim3 grid, hipStream_t st, const u32x4_t *wp,
                        const float *X, int M, int KT, int kpw, int nchunks, int strip0, int nstrips,
                        int n_cols, float *out, int out_stride, size_t chunk_stride) {
  const GemvTopk none{nullptr, nullptr, 0};
  if constexpr (EXACT) {                               // candidate selection: exact slices, <= 8 rows
    if (tk) {
      if (nt)
        hipLaunchKernelGGL((gemv_bf16_kernel<KPW, D, 0, true, EXACT, true>), grid, dim3(GEMV_THREADS), 0, st,
                           wp, X, M, KT, kpw, nchunks, strip0, nstrips, n_cols, out, out_stride,
                           chunk_stride, g_gemv_xcd, *tk);
      else
        hipLaunchKernelGGL((gemv_bf16_kernel<KPW, D, 0, false, EXACT, true>), grid, dim3(GEMV_THREADS), 0, st,
                           wp, X, M, KT, kpw, nchunks, strip0, nstrips, n_cols, out, out_stride,
                           chunk_stride, g_gemv_xcd, *tk);
      return;
    }
  }
#define DART_GEMV_GO(MT_, NT_)                                                                    \
  hipLaunchKernelGGL((gemv_bf16_kernel<KPW, D, MT_, NT_, EXACT>), grid, dim3(GEMV_THREADS), 0, st, \
                     wp, X, M, KT, kpw, nchunks, strip0, nstrips, n_cols, out, out_stride,         \
                     chunk_stride, g_gemv_xcd, none)
  if constexpr (KPW <= 5) {                            // the row-block variants need short k-slices
    if (mt == 4) { if (nt) DART_GEMV_GO(4, true); else DART_GEMV_GO(4, false); return; }
    if (mt == 2) { if (nt) DART_GEMV_GO(2, true); else DART_GEMV_GO(2, false); return; }
  }
  if (mt == 0 && nt) DART_GEMV_GO(0, true);
  else if (mt == 0) DART_GEMV_GO(0, false);
  else if (nt) DART_GEMV_GO(1, true);
  else DART_GEMV_GO(1, false);
#undef DART_GEMV_GO
}

// Number of k-chunks for a matrix with few strips.  With one workgroup per CU, 320 strips of a
// 5120-row matrix leave a quarter of the CUs with twice the work of the rest, and a short
// kernel also pays for each wavefront's activation set-up.  Cutting k into more chunks than
// the register budget demands gives (strip, chunk) units that divide evenly over the CUs and
// shortens the set-up; the consumer adds the extra partials.  Measured on MI355X at d = 5120:
// 7168 rows 25 -> 13 us, 5120 rows 23 -> 11 us, 34816 rows 67 -> 56 us with 4 chunks of 5
// k-steps per wavefront; 5120 rows x 17408 inputs 38 -> 31 us with 17 chunks of 4 k-steps instead
// of 4 chunks of 17; matrices with more than ~12 strips per workgroup (the LM head) gain nothing.
// Only chunk counts that keep every wavefront's k-slice an exact, supported length of at least
// 4 k-steps are used.
DART_TUNABLE int g_gemv_split = 0;      // tuning builds: multiple of the minimum chunk count (0 = automatic)

static bool exact_kpw_supported(int kpw) {
  return kpw == 2 || kpw == 4 || kpw == 5 || kpw == 8 || kpw == 10 || kpw == 12 || kpw == 16 ||
         kpw == 17 || kpw == 20;
}

int gemv_bf16_split(int Kd, int nstrips) {
  const int KT = Kd / 32, base = gemv_bf16_chunks(Kd);
  auto valid = [&](int nch) {
    return KT % (GEMV_WAVES * nch) == 0 && exact_kpw_supported(KT / (GEMV_WAVES * nch));
  };
  if (g_gemv_split > 0) return valid(base * g_gemv_split) ? base * g_gemv_split : base;
  const int wgs_base = max(1, min(g_gemv_wgs_split / base, nstrips));
  if (nstrips / wgs_base >= 12) return base;
  for (int split = 4; split > 1; split /= 2)             // 4 or 2 times the minimum first
    if (valid(base * split) && KT / (GEMV_WAVES * base * split) >= 4) return base * split;
  for (int nch = KT / (GEMV_WAVES * 4); nch > base; --nch)   // else the most chunks of >= 4 k-steps
    if (valid(nch)) return nch;
  return base;
}

// Largest row block (in 16-row tiles) the kernel can take for this matrix cut into nch chunks:
// the activations of a block must fit the register budget next to the weight buffer.
int gemv_bf16_row_tiles(int Kd, int nch) {
  const int KT = Kd / 32;
  if (nch < 1 || KT % (GEMV_WAVES * nch) != 0) return 1;
  const int kpw = KT / (GEMV_WAVES * nch);
  return kpw <= 5 && exact_kpw_supported(kpw) ? 4 : 1;
}

// Launch shape and kernel variant for strips of a matrix, M rows, nch k-chunks.
struct GemvPlan {
  int kpw_t, d_t;       // template k-slice length and rolling-buffer depth
  bool exact, nt;
  int mt, kpw, nchunks, wgs, row_blocks;
};

static hipError_t gemv_plan(const DeviceMatrix &W, int nstrips, int M, int nch, GemvPlan *p) {
  const int KT = W.Kd / 32;
  if (nch < gemv_bf16_chunks(W.Kd)) return hipErrorInvalidValue;
  p->nchunks = nch;
  p->kpw = (KT + GEMV_WAVES * nch - 1) / (GEMV_WAVES * nch);
  p->exact = p->kpw * GEMV_WAVES * nch == KT;
  p->mt = M <= 8 ? 0 : 1;
  p->row_blocks = 1;
  if (M > 16) {
    if (gemv_bf16_row_tiles(W.Kd, nch) < 2) return hipErrorInvalidValue;   // <= 16 rows per launch
    p->mt = M > 32 ? 4 : 2;
    p->row_blocks = (M + 16 * p->mt - 1) / (16 * p->mt);
  }
  int wgs = (nch == 1 ? g_gemv_wgs : g_gemv_wgs_split) / (nch * p->row_blocks);
  p->wgs = max(1, min(wgs, nstrips));
  p->nt = g_gemv_nt && (int64_t)nstrips * KT / 1024 >= g_gemv_nt_min_mb;
  const int depth = g_gemv_depth, kpw = p->kpw;
  const bool m8 = p->mt == 0;
  if (p->exact && exact_kpw_supported(kpw)) {
    p->kpw_t = kpw;
    p->d_t = kpw;
    if (kpw == 20 && (depth == 10 || (depth == 0 && !m8))) p->d_t = 10;
    else if (kpw == 20 && depth == 5) p->d_t = 5;
    else if (kpw == 16 && depth == 8) p->d_t = 8;
  } else {
    p->exact = false;
    p->kpw_t = kpw <= 4 ? 4 : (kpw <= 8 ? 8 : (kpw <= 12 ? 12 : (kpw <= 16 ? 16 : 20)));
    p->d_t = p->kpw_t <= 8 ? p->kpw_t : p->kpw_t / 2;
  }
  return hipSuccess;
}

// "gemv_bf16_kernel<KPW,D,MT,NT,EXACT[,true]> grid=<workgroups>x512" (",true": the candidate-
// selecting variant) of the launch that
// launch_gemv_bf16 makes for these arguments (diagnostics: keys the counter summaries).
int gemv_bf16_describe(const DeviceMatrix &W, int nstrips, int M, int nch, char *buf, int len, bool topk) {
  GemvPlan p;
  if (gemv_plan(W, nstrips, M, nch, &p) != hipSuccess) return -1;
  return snprintf(buf, len, "gemv_bf16_kernel<%d,%d,%d,%s,%s%s> grid=%dx%d", p.kpw_t, p.d_t, p.mt,
                  p.nt ? "true" : "false", p.exact ? "true" : "false", topk ? ",true" : "",
                  p.wgs * p.nchunks * p.row_blocks, GEMV_THREADS);
}

// Strips [strip0, strip0+nstrips) of the packed matrix; out[chunk][m][j], j < nstrips*16
// (columns beyond W.n_real - strip0*16 are not written).  nch: k-chunks (at least
// gemv_bf16_chunks(Kd); 1 when the output must be complete in a single chunk).  M may exceed 16
// only up to 16 * gemv_bf16_row_tiles(Kd, nch) * any number of row blocks (grid.y).
// Workgroups of the launch that computes these strips for M <= 8 rows in one k-chunk, if that
// launch can also select its workgroups' top-k candidates (GemvTopk); 0 if it cannot: the k
// range must be one chunk of exact slices and a workgroup's strips must fit its LDS buffer.
int gemv_bf16_select_wgs(const DeviceMatrix &W, int nstrips, int M) {
  GemvPlan p;
  if (M > 8 || gemv_bf16_chunks(W.Kd) != 1 || gemv_plan(W, nstrips, M, 1, &p) != hipSuccess || !p.exact)
    return 0;
  // strips per workgroup under the kernel's assignment (contiguous eighths of the strips per XCD
  // class when the workgroup count divides by 8, else dealt round-robin)
  const int per_wg = g_gemv_xcd == 2 && p.wgs % 8 == 0
                         ? ((nstrips + 7) / 8 + p.wgs / 8 - 1) / (p.wgs / 8)
                         : (nstrips + p.wgs - 1) / p.wgs;
  return per_wg <= GEMV_TK_STRIPS ? p.wgs : 0;
}

hipError_t launch_gemv_bf16(const DeviceMatrix &W, int strip0, int nstrips, const float *X, int M,
                            float *out, int out_stride, size_t chunk_stride, int nch, int *chunks,
                            hipStream_t st, const GemvTopk *tk) {
  GemvPlan p;
  hipError_t e = gemv_plan(W, nstrips, M, nch, &p);
  if (e != hipSuccess) return e;
  if (tk && (nch != 1 || gemv_bf16_select_wgs(W, nstrips, M) != p.wgs || !tk->cand || !tk->ms))
    return hipErrorInvalidValue;
  const int KT = W.Kd / 32, nchunks = p.nchunks, kpw = p.kpw, mt = p.mt;
  if (chunks) *chunks = nchunks;
  const int n_cols = min(nstrips * 16, W.n_real - strip0 * 16);
  dim3 grid(p.wgs * nchunks, p.row_blocks);
  const u32x4_t *wp = (const u32x4_t *)W.data;
  const bool nt = p.nt;
#define DART_GEMV_ARGS nt, mt, tk, grid, st, wp, X, M, KT, kpw, nchunks, strip0, nstrips, n_cols, out, out_stride, chunk_stride
#define DART_GEMV_CASE(KPW_, D_, EX_) \
  if (p.kpw_t == KPW_ && p.d_t == D_ && p.exact == EX_) gemv_launch<KPW_, D_, EX_>(DART_GEMV_ARGS); else
  DART_GEMV_CASE(20, 20, true) DART_GEMV_CASE(20, 10, true) DART_GEMV_CASE(20, 5, true)
  DART_GEMV_CASE(17, 17, true) DART_GEMV_CASE(16, 16, true) DART_GEMV_CASE(16, 8, true)
  DART_GEMV_CASE(12, 12, true) DART_GEMV_CASE(10, 10, true) DART_GEMV_CASE(8, 8, true)
  DART_GEMV_CASE(5, 5, true) DART_GEMV_CASE(4, 4, true) DART_GEMV_CASE(2, 2, true)
  DART_GEMV_CASE(4, 4, false) DART_GEMV_CASE(8, 8, false) DART_GEMV_CASE(12, 6, false)
  DART_GEMV_CASE(16, 8, false) DART_GEMV_CASE(20, 10, false)
  return hipErrorInvalidValue;
#undef DART_GEMV_CASE
#undef DART_GEMV_ARGS
  return hipGetLastError();
}

}  // namespace dart
