// Multi-row projection on bf16 weights: out[m][n] = sum_k X[m][k] W[n][k] for many rows.
//
// This is the contraction of the batched draft step (e.g. 16 sequences x K = 8 masked
// positions = 128 rows against the LM head, paper Sec. 3.2) and of the K/V build of many
// prefix rows at once.  Every weight is still read from HBM once, but with 128 rows each
// weight byte now feeds 128 FLOP, which only the matrix cores can absorb: the kernel has to
// keep both the HBM stream and the MFMA pipe busy.
//
// Roles: weights are the MFMA A operand, read straight from global memory in the packed tile
// layout (1 KiB per 16 outputs x 32 inputs, already in operand order) -- each tile is used by
// exactly one wavefront, so staging it in LDS would buy nothing.  Activations are the B
// operand, read from a buffer of packed operand tiles (1 KiB per 16 rows x 32 inputs, in operand
// order) in one of two formats: one fp16 tile per row tile against the fp16 copy of the weights
// (contexts of the batched calls: one product per weight tile), or a bf16 hi tile and a bf16 lo
// tile (x ~= hi + lo to 2^-17) against the exact bf16 weights (two products).  The tiles are
// written by whichever kernel produces the rows -- the input norm, the attention merge, the
// residual + norm kernels, the gate/up projection's SwiGLU epilogue -- and only rows that arrive
// as plain fp32 (the FC input of the front end) go through pack_rows_kernel first.  The GEMM
// workgroup copies the tiles of its row block (up to 128 rows) for two k-steps at a time from
// global memory straight into LDS (no registers involved) and its 8 wavefronts share them,
// each applying them to its own strips of 16 outputs.  A wavefront holds up to 5 strips x 8
// row tiles of fp32 accumulators.
//
// Work units: (row block of 16*NCT rows, contiguous strip range, k-chunk).  Strip ranges are
// a balanced partition, so a launch with one range per compute unit has no tail; a range
// longer than 40 strips takes several passes over k.  The sum of a row is one chain per
// k-chunk in k order (hi product, then lo product, per 32-input step), independent of the
// number of rows and of the strip grouping; chunk partials are added by the consumer.
#include <cstdio>
#include <type_traits>

#include "common.h"
#include "dart_internal.h"

namespace dart {

constexpr int GEMM_WAVES = 8;
constexpr int GEMM_THREADS = GEMM_WAVES * 64;
constexpr int GEMM_SMAX = 5;        // strips per wavefront per pass
constexpr int GEMM_KS = 2;          // k-steps (of 32 inputs) per LDS stage = per loop body

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((address_space(3))) void *lptr_t;

// One LDS stage: the operand tiles (TERMS per row tile: hi and lo, or one fp16 tile) of NCT row
// tiles for GEMM_KS k-steps.
template <int NCT, int TERMS>
struct GemmStage {
  u32x4_t t[GEMM_KS][NCT * TERMS][64];
};
// LDS stages in the ring.  A stage is copied GEMM_STAGES - 1 stages before it is read: with one
// stage of lookahead a stage cannot take less than the latency of its copy, which bounds the
// passes with few strips per wavefront (8 KiB of weights per stage and workgroup instead of
// 64) -- the k-chunked projections and the short last pass of the LM head.  The two-term
// format keeps two stages (its tiles are twice as large and static LDS ends at 64 KiB).
template <int TERMS>
constexpr int gemm_stages() { return TERMS == 1 ? 4 : 2; }

// The main loop keeps three kinds of memory traffic in flight at once: weight tiles for the
// next two k-steps (global -> registers), the next stage of activation tiles (global -> LDS,
// bypassing registers) and the LDS reads of the current stage.  The compiler cannot tell which
// LDS stage a global -> LDS copy targets, so with compiler-visible copies it makes the next
// LDS read wait for every outstanding load, the weight prefetch included.  The loads of the
// loop are therefore issued from inline assembly and waited for by count: loads complete in
// issue order, so "at most N outstanding" identifies exactly which ones have landed.
//
// load_tile: 16 bytes per lane from base + off, non-temporal (weights are read once).  The
// destination is a read-write operand so that the value keeps one register from the load to
// the wait that precedes its first use.
__device__ __forceinline__ void load_tile_async(u32x4_t &dst, uint32_t off, const u32x4_t *base) {
  asm volatile("global_load_dwordx4 %0, %1, %2 nt" : "+v"(dst) : "v"(off), "s"(base) : "memory");
}
// One wavefront copies 1 KiB from global memory (lane l: 16 bytes at base + off) to LDS (lane
// l: 16 bytes at lds_base + 16*l); lds_base is wave-uniform.
__device__ __forceinline__ void copy_tile_to_lds_async(uint32_t lds_base, uint32_t off,
                                                       const u32x4_t *base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_base), "v"(off), "s"(base)
               : "memory");
}
// Wait until at most N of the loads above are outstanding; the tiles named here are the ones
// this wait makes valid (the operands tie their first use to the wait).
template <int N, int SP>
__device__ __forceinline__ void wait_tiles(u32x4_t (&t)[SP]) {
  if constexpr (SP == 5)
    asm volatile("s_waitcnt vmcnt(%5)" : "+v"(t[0]), "+v"(t[1]), "+v"(t[2]), "+v"(t[3]), "+v"(t[4]) : "n"(N));
  else if constexpr (SP == 4)
    asm volatile("s_waitcnt vmcnt(%4)" : "+v"(t[0]), "+v"(t[1]), "+v"(t[2]), "+v"(t[3]) : "n"(N));
  else if constexpr (SP == 2)
    asm volatile("s_waitcnt vmcnt(%2)" : "+v"(t[0]), "+v"(t[1]) : "n"(N));
  else
    asm volatile("s_waitcnt vmcnt(%1)" : "+v"(t[0]) : "n"(N));
}

// Packed activations (pack_store8): [k-step][row tile][terms][64 lanes][8 x 16 bit].  Row tiles
// beyond M and, when KT is odd, one extra k-step are zero, so the consumer needs no guards.
__global__ __launch_bounds__(256) void pack_rows_kernel(const float *__restrict__ X, int M, int Kd,
                                                        int ntiles, int ksteps, int terms,
                                                        u32x4_t *__restrict__ Xp) {
  const int item = blockIdx.x * 256 + threadIdx.x;       // (k-step, row tile, lane)
  const int lane = item & 63, tile = (item >> 6) % ntiles, t = (item >> 6) / ntiles;
  if (t >= ksteps) return;
  const int r = tile * 16 + (lane & 15), k = t * 32 + 8 * (lane >> 4);
  uint4 *pk = reinterpret_cast<uint4 *>(Xp);
  if (r < M && k < Kd) {
    const float *src = X + (size_t)r * Kd + k;
    const float4 a = *reinterpret_cast<const float4 *>(src);
    const float4 b = *reinterpret_cast<const float4 *>(src + 4);
    const float x[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
    pack_store8(pk, ntiles, terms, r, k, x);
  } else {
    pack_zero8(pk, ntiles, terms, r, k);
  }
}

struct GemmArgs {
  const u32x4_t *Wp;     // packed weight tiles
  const u32x4_t *Xp;     // packed activations, ntiles row tiles per k-step
  float *out;            // [nchunks][M][out_stride] (EPI 1: [M][out_stride] SwiGLU products)
  uint16_t *out_pack;    // EPI 2: SwiGLU products as one-term operand tiles of the next projection
  int out_ntiles;        //        (row tiles of that operand)
  size_t chunk_stride;
  int M, KT, nchunks, strip0, nstrips, n_cols, ngroups, out_stride;
  int row_blocks, units, ntiles;
};

// EPI 0: store the accumulators.  EPI 1: the strips hold interleaved gate/up features
// (g f, g f+1, u f, u f+1), one group per lane; store silu(g) * u (needs nchunks == 1).
// EPI 2: the same products, written as fp16 straight into the packed operand tiles that the
// down projection reads (a lane's two features are 4 contiguous bytes of a tile).
// TERMS 2: bf16 weights, activations as bf16 hi + lo (two products per tile pair).
// TERMS 1: fp16 weights and fp16 activations (one product).
template <int NCT, int SP, int EPI, int TERMS>
__device__ __forceinline__ void gemm_pass(const GemmArgs &a, GemmStage<NCT, TERMS> *ring, int rb,
                                          int chunk, int k0, int nk, int sfirst, int ns, int wave) {
  constexpr int NS = gemm_stages<TERMS>(), LA = NS - 1;   // ring size, stages of lookahead
  const int lane = threadIdx.x & 63;
  const int kend = k0 + nk;                               // k-steps [k0, kend) of this chunk
  const int nkp = (nk + GEMM_KS - 1) / GEMM_KS * GEMM_KS;  // an odd tail reads the zero k-step

  // weight tiles of this wavefront's strips (absent strips alias the first one: their
  // products are computed and dropped, which keeps the loop free of branches); sfirst and ns
  // are wave-uniform, so the strip bases live in scalar registers and one vector register
  // holds the byte offset of (k-step, lane) for all of them
  const u32x4_t *wrow[SP];
#pragma unroll
  for (int s = 0; s < SP; ++s) {
    const int strip = a.strip0 + sfirst + (s < ns ? s : 0);
    wrow[s] = a.Wp + (size_t)strip * a.KT * 64;
  }
  auto tile_off = [&](int kstep) { return (uint32_t)(min(kstep, kend - 1) * 64 + lane) * 16u; };

  // stage copy: the NCT*TERMS operand tiles of GEMM_KS k-steps, 1 KiB each; wavefront w moves
  // tiles w, w+8, ...: exactly TPW copies per wavefront and stage (with fewer tiles than
  // wavefronts some tiles are copied twice, so that every wavefront counts the same)
  constexpr int NT = GEMM_KS * NCT * TERMS;
  static_assert(NT % GEMM_WAVES == 0 || GEMM_WAVES % NT == 0, "uniform copies per wavefront");
  constexpr int TPW = NT >= GEMM_WAVES ? NT / GEMM_WAVES : 1;
  const u32x4_t *xbase = a.Xp + (size_t)rb * NCT * 64 * TERMS;   // uniform
  const uint32_t xstep = (uint32_t)a.ntiles * 1024u * TERMS;     // bytes of one k-step
  auto stage_copy = [&](int kstage, GemmStage<NCT, TERMS> *dst) {   // kstage: first k-step, absolute
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
      const int tile = (wave + GEMM_WAVES * i) % NT;
      const int u = tile / (NCT * TERMS), c2 = tile % (NCT * TERMS);
      copy_tile_to_lds_async((uint32_t)(uintptr_t)(lptr_t)&dst->t[u][c2][0],
                             (uint32_t)(kstage + u) * xstep + (uint32_t)(c2 * 64 + lane) * 16u, xbase);
    }
  };

  f32x4_t acc[SP][NCT];
#pragma unroll
  for (int s = 0; s < SP; ++s)
#pragma unroll
    for (int c = 0; c < NCT; ++c) acc[s][c] = {0.f, 0.f, 0.f, 0.f};

  // Ring of weight tiles: PD k-steps deep, slot t % PD serves k-step t and is refilled (with
  // k-step t + PD) right after the products that consumed it.  8 to 16 KiB are in flight per
  // wavefront (64 to 128 KiB per compute unit) whatever the number of strips, so that neither
  // the full passes nor the ones with few strips per wavefront are bound by memory latency.
  // Five strips per wavefront (one pass over k for up to 40 strips per workgroup: the LM head's
  // 37-38 at 256 workgroups, which otherwise pays the staging of all operand tiles a second
  // time for 5-6 left-over strips) leave registers for a ring of two k-steps (10 KiB in flight)
  // and for two operand tiles at a time.
  constexpr int PD = SP == 5 ? 2 : (SP == 4 ? 4 : 8 / SP);
  // k-steps per unrolled loop body: a multiple of the weight ring and of the stage ring, so
  // that both kinds of slot are static
  constexpr int UNR = NS == 4 ? 8 : (PD < 4 ? 4 : PD);
  static_assert(UNR % PD == 0 && (UNR / GEMM_KS) % NS == 0, "static ring slots");
  u32x4_t aop[PD][SP];
  // prologue: the first LA stages, then the weight tiles of the first PD k-steps, issued in
  // the same pattern as the loop issues them (per stage: copies, then two k-steps of tiles;
  // the copies of that pattern just repeat the last of the LA stages), so that the counted
  // waits below hold from the first k-step on
  const int klast = k0 + nkp - GEMM_KS;                   // first k-step of the last stage
#pragma unroll
  for (int j = 0; j < LA; ++j) stage_copy(min(k0 + j * GEMM_KS, klast), &ring[j]);
#pragma unroll
  for (int p = 0; p < PD; ++p) {
    if (p % GEMM_KS == 0) stage_copy(min(k0 + (LA - 1) * GEMM_KS, klast), &ring[LA - 1]);
#pragma unroll
    for (int s = 0; s < SP; ++s) {
      aop[p][s] = u32x4_t{0, 0, 0, 0};
      load_tile_async(aop[p][s], tile_off(k0 + p), wrow[s]);
    }
  }
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(GEMM_KS * SP) : "memory");

  // One stage: GEMM_KS k-steps out of ring slot `cur` while the stage LA stages ahead is copied
  // into the slot that the previous stage has just left; J is the position of the stage's first
  // k-step in the unrolled body (ring slots are static).
  auto stage_body = [&](int t0, auto jtag) {
    constexpr int J = decltype(jtag)::value;
    GemmStage<NCT, TERMS> *cur = &ring[(J / GEMM_KS) % NS];
    // (clamped at the end: the last stage is copied again, into a slot that is not read any more)
    stage_copy(min(k0 + t0 + LA * GEMM_KS, klast), &ring[(J / GEMM_KS + LA) % NS]);
#pragma unroll
    for (int u = 0; u < GEMM_KS; ++u) {
      const int slot = (J + u) % PD;
      // Issued after this k-step's tiles and possibly still in flight: the tiles of the PD - 1
      // following k-steps and the stage copies of the PD / 2 stage starts since then.
      wait_tiles<(PD - 1) * SP + (PD / 2) * TPW, SP>(aop[slot]);
      // operand tiles are read NB at a time (registers), hi then lo of each row tile: every
      // accumulator still adds its hi product, then its lo product, k-step by k-step
      constexpr int NB = SP == 5 ? 2 : (NCT < 4 ? NCT : 4);
#pragma unroll
      for (int cb = 0; cb < NCT; cb += NB) {
#pragma unroll
        for (int hl = 0; hl < TERMS; ++hl) {
          u32x4_t b[NB];
#pragma unroll
          for (int c = 0; c < NB; ++c) b[c] = cur->t[u][TERMS * (cb + c) + hl][lane];
#pragma unroll
          for (int s = 0; s < SP; ++s) {
#pragma unroll
            for (int c = 0; c < NB; ++c) {
              if constexpr (TERMS == 2)
                acc[s][cb + c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                    __builtin_bit_cast(bf16x8_t, aop[slot][s]), __builtin_bit_cast(bf16x8_t, b[c]),
                    acc[s][cb + c], 0, 0, 0);
              else
                acc[s][cb + c] = __builtin_amdgcn_mfma_f32_16x16x32_f16(
                    __builtin_bit_cast(f16x8_t, aop[slot][s]), __builtin_bit_cast(f16x8_t, b[c]),
                    acc[s][cb + c], 0, 0, 0);
            }
          }
        }
      }
      // refill the ring slot just consumed (clamped: reloads of the last tile are never used)
      const uint32_t off = tile_off(k0 + t0 + u + PD);
#pragma unroll
      for (int s = 0; s < SP; ++s) load_tile_async(aop[slot][s], off, wrow[s]);
      // keep the k-steps apart: hoisting the next step's operand reads over this step's
      // products would need more registers than a wavefront has
      __builtin_amdgcn_sched_barrier(0);
    }
    // The next stage was copied LA stage starts ago.  Issued since then, oldest first: the
    // refills of LA stages (GEMM_KS * SP each) and the copies of the LA - 1 later stage starts
    // (TPW each): once at most that many loads remain, this wavefront's part of the next stage
    // is in LDS and the barrier publishes it; the weight prefetch and the copies of the stages
    // after it stay in flight
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(LA * GEMM_KS * SP + (LA - 1) * TPW)
                 : "memory");
  };
  for (int t0 = 0; t0 < nkp; t0 += UNR) {
    stage_body(t0, std::integral_constant<int, 0>{});
    if (t0 + 2 < nkp) stage_body(t0 + 2, std::integral_constant<int, 2>{});
    if constexpr (UNR == 8) {
      if (t0 + 4 < nkp) stage_body(t0 + 4, std::integral_constant<int, 4>{});
      if (t0 + 6 < nkp) stage_body(t0 + 6, std::integral_constant<int, 6>{});
    }
  }
  // the clamped refills and the last stage copy are still in flight: let them land before the
  // registers and the LDS stages are reused
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

  // D[i][j] of a tile: output i = 4*(lane/16) + reg of the strip, row j = lane%16 of the tile
  const int j = lane & 15, i4 = (lane >> 4) * 4;
  const int m0 = rb * 16 * NCT;
#pragma unroll
  for (int s = 0; s < SP; ++s) {
    if (s < ns) {
      const int col = (sfirst + s) * 16 + i4;
#pragma unroll
      for (int c = 0; c < NCT; ++c) {
        const int m = m0 + 16 * c + j;
        if (m < a.M) {
          const f32x4_t v = acc[s][c];
          if constexpr (EPI != 0) {
            if (col < a.n_cols) {
              const float h0 = v[0] / (1.0f + expf(-v[0])) * v[2];
              const float h1 = v[1] / (1.0f + expf(-v[1])) * v[3];
              const int f = col >> 1;                    // first of the lane's two features
              if constexpr (EPI == 1) {
                *reinterpret_cast<float2 *>(a.out + (size_t)m * a.out_stride + f) = make_float2(h0, h1);
              } else {
                // element (row m, input f) of the one-term layout (pack_store8)
                uint16_t *dst = a.out_pack +
                                (((size_t)(f >> 5) * a.out_ntiles + (m >> 4)) * 64 +
                                 (((f & 31) >> 3) * 16 + (m & 15))) * 8 + (f & 7);
                *reinterpret_cast<uint32_t *>(dst) =
                    (uint32_t)f32_to_f16_sat_bits(h0) | ((uint32_t)f32_to_f16_sat_bits(h1) << 16);
              }
            }
          } else {
            float *dst = a.out + chunk * a.chunk_stride + (size_t)m * a.out_stride + col;
            if (col + 3 < a.n_cols && (a.out_stride & 3) == 0) {
              *reinterpret_cast<float4 *>(dst) = make_float4(v[0], v[1], v[2], v[3]);
            } else {
#pragma unroll
              for (int r = 0; r < 4; ++r)
                if (col + r < a.n_cols) dst[r] = v[r];
            }
          }
        }
      }
    }
  }
}

template <int NCT, int EPI, int TERMS>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_bf16_kernel(GemmArgs a) {
  __shared__ GemmStage<NCT, TERMS> ring[gemm_stages<TERMS>()];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int gc_count = a.ngroups * a.nchunks;
  for (int unit = blockIdx.x; unit < a.units; unit += gridDim.x) {
    // row blocks of one (group, chunk) sit 8 units apart: same XCD, about the same time, so
    // the second reader of a weight tile finds it in that XCD's L2.
    // Units are dealt to the 8 XCDs round-robin (unit u runs on XCD u % 8): XCD x owns a
    // contiguous eighth of the (group, chunk) pairs, so that each L2 streams one region.
    const int blk = unit / (8 * a.row_blocks), within = unit % (8 * a.row_blocks);
    const int rb = within / 8, x = within % 8, per_x = (gc_count + 7) / 8;
    const int gc = x * per_x + blk;
    if (blk >= per_x || gc >= gc_count) continue;
    const int group = gc / a.nchunks, chunk = gc % a.nchunks;
    const int g0 = (int)((int64_t)a.nstrips * group / a.ngroups);
    const int g1 = (int)((int64_t)a.nstrips * (group + 1) / a.ngroups);
    const int k0 = gemm_chunk_begin(a.KT, a.nchunks, chunk);
    const int nk = gemm_chunk_begin(a.KT, a.nchunks, chunk + 1) - k0;
    for (int base = g0; base < g1; base += GEMM_WAVES * GEMM_SMAX) {
      const int P = min(g1 - base, GEMM_WAVES * GEMM_SMAX);
      const int per = (P + GEMM_WAVES - 1) / GEMM_WAVES;          // strips per wavefront
      const int sfirst = min(base + wave * per, g1 - 1);
      const int ns = max(0, min(per, P - wave * per));
      if (per > 4) gemm_pass<NCT, 5, EPI, TERMS>(a, ring, rb, chunk, k0, nk, sfirst, ns, wave);
      else if (per > 2) gemm_pass<NCT, 4, EPI, TERMS>(a, ring, rb, chunk, k0, nk, sfirst, ns, wave);
      else if (per == 2) gemm_pass<NCT, 2, EPI, TERMS>(a, ring, rb, chunk, k0, nk, sfirst, ns, wave);
      else gemm_pass<NCT, 1, EPI, TERMS>(a, ring, rb, chunk, k0, nk, sfirst, ns, wave);
    }
  }
}

// ---- Many-row projection that reproduces the skinny kernel's sums bit for bit ----
//
// The K/V build of a long prefix (a cold call: thousands of rows against Wk, Wv; Sec. 3.2) must
// leave in the K/V buffers exactly what a later warm call would compute for the same row with
// the skinny kernel, since cached rows and new rows are mixed freely.  The skinny kernel's sum
// for an output element is, per k-chunk, eight k-slices (one per wavefront) of `kpw` k-steps,
// each slice one chain of hi products and one chain of lo products starting from zero; the
// slices' hi sums and lo sums are added in slice order, then hi + lo, and the consumer adds the
// chunks in order.  Here one wavefront owns an output tile for the whole k range and walks the
// slices one after the other: slice accumulators (hi, lo) are flushed into chunk totals every
// kpw k-steps, chunk totals into the final sum every 8 kpw k-steps, each in the same order of
// additions.  The same MFMA with the same operands in the same chain gives the same bits, so
// the result equals the skinny kernel's (tests compare cold and warm calls bit for bit).  No
// partial sums leave the kernel.
//
// A workgroup takes 64 rows (4 row tiles) x 16 strips (2 per wavefront): 20 accumulator
// registers per (strip, row tile) pair fit that shape; the activations (two-term packed tiles)
// go through the same LDS ring as above, the weights stream from L2 (units that share strips
// run on one XCD at the same time).
template <int NCT, int SP>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_ordered_kernel(GemmArgs a, int kpw, int map) {
  // ring of four LDS stages (16 KiB each at 4 row tiles): a stage is copied three stages before
  // it is read, so a stage may take less time than the latency of its copy
  constexpr int TERMS = 2, NS = 4, LA = NS - 1;
  static_assert(sizeof(GemmStage<NCT, TERMS>) * NS <= 64 * 1024, "static LDS");
  __shared__ GemmStage<NCT, TERMS> ring[NS];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  // unit -> (strip group, row block): all row blocks of a strip group run on one XCD (unit u
  // runs on XCD u % 8), so that XCD's L2 serves the group's weights to every one of them
  int group, rb;
  {
    const int u = blockIdx.x, x = u % 8, j = u / 8;
    if (map == 1) {            // XCD x: row blocks x, x + 8, ..., the strip groups of one together
      rb = x + 8 * (j / a.ngroups);
      group = j % a.ngroups;
    } else if (map == 0) {     // XCD x: strip groups x, x + 8, ..., the row blocks of one together
      group = x + 8 * (j / a.row_blocks);
      rb = j % a.row_blocks;
    } else {
      group = u / a.row_blocks;
      rb = u % a.row_blocks;
    }
  }
  if (group >= a.ngroups || rb >= a.row_blocks) return;
  const int g0 = group * GEMM_WAVES * SP, g1 = min(a.nstrips, g0 + GEMM_WAVES * SP);
  const int P = g1 - g0;
  const int per = (P + GEMM_WAVES - 1) / GEMM_WAVES;              // strips per wavefront (<= SP)
  const int sfirst = min(g0 + wave * per, g1 - 1);
  const int ns = max(0, min(per, P - wave * per));
  const int KT = a.KT;                                             // even, = nchunks * 8 * kpw

  const u32x4_t *wrow[SP];
#pragma unroll
  for (int s = 0; s < SP; ++s) {
    const int strip = a.strip0 + sfirst + (s < ns ? s : 0);
    wrow[s] = a.Wp + (size_t)strip * KT * 64;
  }
  auto tile_off = [&](int kstep) { return (uint32_t)(min(kstep, KT - 1) * 64 + lane) * 16u; };
  constexpr int NT = GEMM_KS * NCT * TERMS;
  static_assert(NT % GEMM_WAVES == 0, "uniform copies per wavefront");
  constexpr int TPW = NT / GEMM_WAVES;
  const u32x4_t *xbase = a.Xp + (size_t)rb * NCT * 64 * TERMS;
  const uint32_t xstep = (uint32_t)a.ntiles * 1024u * TERMS;
  auto stage_copy = [&](int kstage, GemmStage<NCT, TERMS> *dst) {
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
      const int tile = wave + GEMM_WAVES * i;
      const int u = tile / (NCT * TERMS), c2 = tile % (NCT * TERMS);
      copy_tile_to_lds_async((uint32_t)(uintptr_t)(lptr_t)&dst->t[u][c2][0],
                             (uint32_t)(kstage + u) * xstep + (uint32_t)(c2 * 64 + lane) * 16u, xbase);
    }
  };

  // slice accumulators, chunk totals, final sums
  f32x4_t ahi[SP][NCT], alo[SP][NCT], thi[SP][NCT], tlo[SP][NCT], sum[SP][NCT];
  const f32x4_t zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int s = 0; s < SP; ++s)
#pragma unroll
    for (int c = 0; c < NCT; ++c) ahi[s][c] = alo[s][c] = thi[s][c] = tlo[s][c] = sum[s][c] = zero;

  constexpr int PD = 8 / SP;                 // weight ring depth in k-steps
  constexpr int UNR = 8;                     // k-steps per unrolled body (multiple of PD and of the stage ring)
  static_assert(UNR % PD == 0 && (UNR / GEMM_KS) % NS == 0, "static ring slots");
  u32x4_t aop[PD][SP];
  const int klast = KT - GEMM_KS;
  // prologue: the first LA stages, then the weight tiles of the first PD k-steps in the pattern
  // the loop issues them (the copies of that pattern just repeat the last of the LA stages), so
  // that the counted waits hold from the first k-step on
#pragma unroll
  for (int j = 0; j < LA; ++j) stage_copy(min(j * GEMM_KS, klast), &ring[j]);
#pragma unroll
  for (int p = 0; p < PD; ++p) {
    if (p % GEMM_KS == 0) stage_copy(min((LA - 1) * GEMM_KS, klast), &ring[LA - 1]);
#pragma unroll
    for (int s = 0; s < SP; ++s) {
      aop[p][s] = u32x4_t{0, 0, 0, 0};
      load_tile_async(aop[p][s], tile_off(p), wrow[s]);
    }
  }
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(GEMM_KS * SP) : "memory");

  int in_slice = 0, in_chunk = 0;            // k-steps done of the current slice / slices of the chunk
  auto stage_body = [&](int t0, auto jtag) {
    constexpr int J = decltype(jtag)::value;
    GemmStage<NCT, TERMS> *cur = &ring[(J / GEMM_KS) % NS];
    stage_copy(min(t0 + LA * GEMM_KS, klast), &ring[(J / GEMM_KS + LA) % NS]);
#pragma unroll
    for (int u = 0; u < GEMM_KS; ++u) {
      const int slot = (J + u) % PD;
      wait_tiles<(PD - 1) * SP + (PD / 2) * TPW, SP>(aop[slot]);
#pragma unroll
      for (int hl = 0; hl < TERMS; ++hl) {
        u32x4_t b[NCT];
#pragma unroll
        for (int c = 0; c < NCT; ++c) b[c] = cur->t[u][TERMS * c + hl][lane];
#pragma unroll
        for (int s = 0; s < SP; ++s)
#pragma unroll
          for (int c = 0; c < NCT; ++c) {
            f32x4_t &acc = hl == 0 ? ahi[s][c] : alo[s][c];
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, aop[slot][s]),
                                                          __builtin_bit_cast(bf16x8_t, b[c]), acc, 0, 0, 0);
          }
      }
      const uint32_t off = tile_off(t0 + u + PD);
#pragma unroll
      for (int s = 0; s < SP; ++s) load_tile_async(aop[slot][s], off, wrow[s]);
      // end of a k-slice: its sums join the chunk totals (hi and lo apart, slice order); end of
      // a k-chunk: hi + lo joins the final sum (chunk order).  Uniform branches, no memory.
      if (++in_slice == kpw) {
        in_slice = 0;
#pragma unroll
        for (int s = 0; s < SP; ++s)
#pragma unroll
          for (int c = 0; c < NCT; ++c) {
            thi[s][c] += ahi[s][c];
            tlo[s][c] += alo[s][c];
            ahi[s][c] = zero;
            alo[s][c] = zero;
          }
        if (++in_chunk == GEMM_WAVES) {
          in_chunk = 0;
#pragma unroll
          for (int s = 0; s < SP; ++s)
#pragma unroll
            for (int c = 0; c < NCT; ++c) {
              sum[s][c] += thi[s][c] + tlo[s][c];
              thi[s][c] = zero;
              tlo[s][c] = zero;
            }
        }
      }
    }
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(LA * GEMM_KS * SP + (LA - 1) * TPW)
                 : "memory");
  };
  for (int t0 = 0; t0 < KT; t0 += UNR) {
    stage_body(t0, std::integral_constant<int, 0>{});
    if (t0 + 2 < KT) stage_body(t0 + 2, std::integral_constant<int, 2>{});
    if constexpr (UNR == 8) {
      if (t0 + 4 < KT) stage_body(t0 + 4, std::integral_constant<int, 4>{});
      if (t0 + 6 < KT) stage_body(t0 + 6, std::integral_constant<int, 6>{});
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

  const int j = lane & 15, i4 = (lane >> 4) * 4;
  const int m0 = rb * 16 * NCT;
#pragma unroll
  for (int s = 0; s < SP; ++s) {
    if (s < ns) {
      const int col = (sfirst + s) * 16 + i4;
#pragma unroll
      for (int c = 0; c < NCT; ++c) {
        const int m = m0 + 16 * c + j;
        if (m < a.M) {
          const f32x4_t v = sum[s][c];
          float *dst = a.out + (size_t)m * a.out_stride + col;
          if (col + 3 < a.n_cols && (a.out_stride & 3) == 0) {
            *reinterpret_cast<float4 *>(dst) = make_float4(v[0], v[1], v[2], v[3]);
          } else {
#pragma unroll
            for (int r = 0; r < 4; ++r)
              if (col + r < a.n_cols) dst[r] = v[r];
          }
        }
      }
    }
  }
}

// fp16 copy of a matrix of packed bf16 tiles (same tile layout: both are 16-bit operands of a
// 16x16x32 MFMA).  bf16 -> fp16 is exact for 2^-14 <= |w| < 65520; smaller weights round to
// fp16 subnormals (absolute error <= 2^-25), larger ones saturate.
__global__ __launch_bounds__(256) void tiles_to_f16_kernel(const uint32_t *__restrict__ src,
                                                           uint32_t *__restrict__ dst, size_t n_pairs) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n_pairs; i += (size_t)gridDim.x * 256) {
    const uint32_t v = src[i];
    const float lo = bf16_to_f32((bf16_t)(v & 0xFFFF)), hi = bf16_to_f32((bf16_t)(v >> 16));
    dst[i] = (uint32_t)f32_to_f16_sat_bits(lo) | ((uint32_t)f32_to_f16_sat_bits(hi) << 16);
  }
}
hipError_t launch_tiles_to_f16(const void *src, void *dst, size_t n_elems, hipStream_t st) {
  hipLaunchKernelGGL(tiles_to_f16_kernel, dim3(2048), dim3(256), 0, st, (const uint32_t *)src,
                     (uint32_t *)dst, n_elems / 2);
  return hipGetLastError();
}

DART_TUNABLE int g_gemm_wgs = 256;      // resident workgroups: one per compute unit
DART_TUNABLE int g_gemm_ord_map = 1;    // unit-to-XCD map of gemm_ordered_kernel, see there

// k-chunks of a matrix on this path: fixed per matrix so that a row's sums do not depend on
// the call.  Matrices with few strips are cut along k until (strip ranges of 8 strips, one per
// wavefront) x chunks fill the compute units; chunks are at least 16 k-steps long.  Narrow
// ranges keep the chunk count, and with it the fp32 partial sums written here and read back by
// the next kernel, small: at 128 rows a chunk of partials is a quarter of the O projection's
// weights.
int gemm_bf16_chunks(int Kd, int nstrips) {
  const int KT = Kd / 32;
  const int groups = (nstrips + GEMM_WAVES - 1) / GEMM_WAVES;
  if (groups >= g_gemm_wgs / 2) return 1;
  int nch = g_gemm_wgs / groups;          // rounded down: one more unit than workgroups costs a second round
  nch = min(nch, max(1, KT / 16));
  return max(1, nch);
}

// Row tiles the packed activations of M rows hold (whole row blocks of the kernel variant
// that M selects) and their size in bytes.
static int gemm_nct(int M) { return M <= 32 ? 2 : (M <= 64 ? 4 : 8); }
void gemm_bf16_pack_shape(int M, int Kd, int *ntiles, int *ksteps) {
  const int nct = gemm_nct(M);
  *ntiles = (M + 16 * nct - 1) / (16 * nct) * nct;
  *ksteps = (Kd / 32 + 1) / 2 * 2;
}
size_t gemm_bf16_pack_bytes(int M, int Kd) {      // of the larger (two-term) format
  const int nct = gemm_nct(M), ntiles = (M + 16 * nct - 1) / (16 * nct) * nct;
  const int ksteps = (Kd / 32 + 1) / 2 * 2;
  return (size_t)ksteps * ntiles * 2048;
}

// The matrix's fp16 copy, when it has one, selects the one-term arithmetic (fp16 activations);
// the packed activations must be in the matching format (gemm_bf16_terms).
int gemm_bf16_terms(const DeviceMatrix &W) { return W.data16 ? 1 : 2; }

// Row tiling and grid of a launch (shared with the diagnostic description below).
static void gemm_shape(int nstrips, int M, int nchunks, GemmArgs *a, int *nct_out) {
  const int nct = gemm_nct(M);
  a->row_blocks = (M + 16 * nct - 1) / (16 * nct);
  a->ntiles = a->row_blocks * nct;
  // strip ranges: as many as fill the machine, but at least one strip per wavefront
  const int groups_max = (nstrips + GEMM_WAVES - 1) / GEMM_WAVES;
  a->ngroups = max(1, min(groups_max, g_gemm_wgs / (nchunks * a->row_blocks)));
  const int gc = a->ngroups * nchunks;
  a->units = (gc + 7) / 8 * 8 * a->row_blocks;
  *nct_out = nct;
}

// "gemm_bf16_kernel<NCT,EPI,TERMS> grid=<workgroups>x512" of the launch that launch_gemm_bf16
// makes for these arguments (diagnostics: keys the counter summaries).
int gemm_bf16_describe(const DeviceMatrix &W, int nstrips, int M, int nchunks, int epi, char *buf,
                       int len) {
  GemmArgs a;
  int nct = 0;
  gemm_shape(nstrips, M, nchunks, &a, &nct);
  const int per_range = (nstrips + a.ngroups - 1) / a.ngroups;      // strips of the longest range
  const int passes = (per_range + GEMM_WAVES * GEMM_SMAX - 1) / (GEMM_WAVES * GEMM_SMAX);
  return snprintf(buf, len, "gemm_bf16_kernel<%d,%d,%d> grid=%dx%d strips/wg=%d passes=%d", nct, epi,
                  gemm_bf16_terms(W), a.units, GEMM_THREADS, per_range, passes);
}

// fp32 rows X[M][Kd] -> packed operand tiles (gemm_bf16_pack_shape(M, Kd) row tiles; terms 2: bf16
// hi + lo with the skinny kernel's split, terms 1: fp16).
hipError_t launch_pack_rows(const float *X, int M, int Kd, int terms, void *pack, hipStream_t st) {
  if (!X || !pack || M < 1 || Kd < 32 || (terms != 1 && terms != 2)) return hipErrorInvalidValue;
  int ntiles = 0, ksteps = 0;
  gemm_bf16_pack_shape(M, Kd, &ntiles, &ksteps);
  const int64_t items = (int64_t)ksteps * ntiles * 64;
  hipLaunchKernelGGL(pack_rows_kernel, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, st, X, M, Kd,
                     ntiles, ksteps, terms, (u32x4_t *)pack);
  return hipGetLastError();
}

hipError_t launch_gemm_bf16(const DeviceMatrix &W, int strip0, int nstrips, const float *X, int M,
                            void *pack, float *out, int out_stride, size_t chunk_stride, int nchunks,
                            int epi, hipStream_t st, void *out_pack) {
  if (M < 1 || nstrips < 1 || nchunks < 1 || (epi != 0 && nchunks != 1)) return hipErrorInvalidValue;
  const int terms = gemm_bf16_terms(W);
  if (epi == 2 && (!out_pack || terms != 1)) return hipErrorInvalidValue;
  GemmArgs a;
  a.Wp = (const u32x4_t *)(terms == 1 ? W.data16 : W.data);
  a.Xp = (const u32x4_t *)pack;
  a.out = out;
  a.chunk_stride = chunk_stride;
  a.M = M;
  a.KT = W.Kd / 32;
  a.nchunks = nchunks;
  a.strip0 = strip0;
  a.nstrips = nstrips;
  a.n_cols = min(nstrips * 16, W.n_real - strip0 * 16);
  a.out_stride = out_stride;
  int nct = 0;
  gemm_shape(nstrips, M, nchunks, &a, &nct);
  a.out_pack = (uint16_t *)out_pack;
  a.out_ntiles = a.ntiles;                // the next projection carries the same rows
  const int ksteps = (a.KT + 1) / 2 * 2;
  if (X) {                                               // X == nullptr: pack already holds them
    hipError_t e = launch_pack_rows(X, M, W.Kd, terms, pack, st);
    if (e != hipSuccess) return e;
  }
  const dim3 grid(a.units), block(GEMM_THREADS);
#define DART_GEMM_GO(NCT_)                                                                        \
  do {                                                                                            \
    if (terms == 1) {                                                                             \
      if (epi == 2) hipLaunchKernelGGL((gemm_bf16_kernel<NCT_, 2, 1>), grid, block, 0, st, a);    \
      else if (epi == 1) hipLaunchKernelGGL((gemm_bf16_kernel<NCT_, 1, 1>), grid, block, 0, st, a); \
      else hipLaunchKernelGGL((gemm_bf16_kernel<NCT_, 0, 1>), grid, block, 0, st, a);             \
    } else {                                                                                      \
      if (epi == 1) hipLaunchKernelGGL((gemm_bf16_kernel<NCT_, 1, 2>), grid, block, 0, st, a);    \
      else hipLaunchKernelGGL((gemm_bf16_kernel<NCT_, 0, 2>), grid, block, 0, st, a);             \
    }                                                                                             \
  } while (0)
  if (nct == 2) DART_GEMM_GO(2);
  else if (nct == 4) DART_GEMM_GO(4);
  else DART_GEMM_GO(8);
#undef DART_GEMM_GO
  return hipGetLastError();
}

// Can the order-preserving many-row kernel serve this matrix cut into nch k-chunks of the skinny
// kernel?  It needs whole k-slices (KT = nch * 8 * kpw) and an even number of k-steps.
bool gemm_ordered_supported(const DeviceMatrix &W, int nch) {
  const int KT = W.Kd / 32;
  return nch >= 1 && KT % 2 == 0 && KT % (GEMM_WAVES * nch) == 0 && KT >= 8;
}

// out[m][j] (row stride out_stride) = the skinny kernel's result for strips [strip0, strip0+nstrips)
// of W with nch k-chunks, chunk partials already added; pack: two-term operand tiles of the M rows
// (gemm_bf16_pack_shape(M, Kd) row tiles, written by the input norm).
hipError_t launch_gemm_ordered(const DeviceMatrix &W, int strip0, int nstrips, int M, const void *pack,
                               float *out, int out_stride, int nch, hipStream_t st) {
  if (M < 1 || nstrips < 1 || !gemm_ordered_supported(W, nch)) return hipErrorInvalidValue;
  constexpr int NCT = 4, SP = 2;
  GemmArgs a{};
  a.Wp = (const u32x4_t *)W.data;
  a.Xp = (const u32x4_t *)pack;
  a.out = out;
  a.M = M;
  a.KT = W.Kd / 32;
  a.strip0 = strip0;
  a.nstrips = nstrips;
  a.n_cols = min(nstrips * 16, W.n_real - strip0 * 16);
  a.out_stride = out_stride;
  int ntiles = 0, ksteps = 0;
  gemm_bf16_pack_shape(M, W.Kd, &ntiles, &ksteps);
  if (ntiles % NCT != 0) return hipErrorInvalidValue;
  a.ntiles = ntiles;
  a.row_blocks = (M + 16 * NCT - 1) / (16 * NCT);
  a.ngroups = (nstrips + GEMM_WAVES * SP - 1) / (GEMM_WAVES * SP);
  int map = g_gemm_ord_map;
  if (map == 1) a.units = 8 * ((a.row_blocks + 7) / 8) * a.ngroups;
  else if (map == 0) a.units = 8 * ((a.ngroups + 7) / 8) * a.row_blocks;
  else a.units = a.ngroups * a.row_blocks;
  const int kpw = a.KT / (GEMM_WAVES * nch);
  hipLaunchKernelGGL((gemm_ordered_kernel<NCT, SP>), dim3(a.units), dim3(GEMM_THREADS), 0, st, a, kpw, map);
  return hipGetLastError();
}

}  // namespace dart
