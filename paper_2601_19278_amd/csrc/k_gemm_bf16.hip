// Multi-row projection on bf16 weights: out[m][n] = sum_k X[m][k] W[n][k] for M > 16 rows.
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
// operand: a block of up to 128 rows is converted once per workgroup from fp32 to bf16
// hi + lo parts (x ~= hi + lo to 2^-17, weights stay the exact bf16 values), written to LDS
// in operand order, and shared by the 4 wavefronts (one per SIMD, so that each can hold
// 8 strips x 8 row tiles of fp32 accumulators = 256 registers next to its operands), each of
// which applies it to its own strips of 16 outputs.
//
// Work units: (row block of 16*NCT rows, contiguous strip range, k-chunk).  Strip ranges are
// a balanced partition, so a launch with one range per compute unit has no tail; a range
// longer than 32 strips takes several passes over k.  The sum of a row is one chain per
// k-chunk in k order (hi product, then lo product, per 32-input step), independent of the
// number of rows and of the strip grouping; chunk partials are added by the consumer.
#include "common.h"
#include "dart_internal.h"

namespace dart {

constexpr int GEMM_WAVES = 4;       // one wavefront per SIMD: each may use the full 512 registers
constexpr int GEMM_THREADS = GEMM_WAVES * 64;
constexpr int GEMM_SMAX = 8;        // strips per wavefront per pass
constexpr int GEMM_KS = 2;          // k-steps (of 32 inputs) per LDS stage
constexpr int GEMM_PD = 2;          // k-steps of weight tiles in flight per wavefront
constexpr int GEMM_UNR = 2;         // k-steps per loop body: one LDS stage, one turn of the ring

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

__device__ __forceinline__ void gemm_lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

struct GemmArgs {
  const u32x4_t *Wp;     // packed weight tiles
  const float *X;        // [M][Kd]
  float *out;            // [nchunks][M][out_stride] (EPI 1: [M][out_stride] SwiGLU products)
  size_t chunk_stride;
  int M, KT, nchunks, strip0, nstrips, n_cols, ngroups, out_stride;
  int row_blocks, units;
};

// EPI 0: store the accumulators.  EPI 1: the strips hold interleaved gate/up features
// (g f, g f+1, u f, u f+1), one group per lane; store silu(g) * u (needs nchunks == 1).
template <int NCT, int SP, int EPI>
__device__ __forceinline__ void gemm_pass(const GemmArgs &a, u32x4_t (*bst)[GEMM_KS][NCT * 2][64],
                                          int m0, int chunk, int k0, int nk, int sfirst, int ns) {
  const int lane = threadIdx.x & 63;
  const int Kd = a.KT * 32;
  const int kend = k0 + nk;                               // k-steps [k0, kend) of this chunk
  const int nkp = (nk + GEMM_UNR - 1) / GEMM_UNR * GEMM_UNR;

  // weight tile pointers of this wavefront's strips (absent strips alias the first one: their
  // products are computed and dropped, which keeps the loop free of branches)
  // (sfirst and ns are wave-uniform, so these pointers live in scalar registers)
  const u32x4_t *wrow[SP];
#pragma unroll
  for (int s = 0; s < SP; ++s) {
    const int strip = a.strip0 + sfirst + (s < ns ? s : 0);
    wrow[s] = a.Wp + (size_t)strip * a.KT * 64;
  }
  u32x4_t aop[GEMM_PD][SP];
#pragma unroll
  for (int p = 0; p < GEMM_PD; ++p)
#pragma unroll
    for (int s = 0; s < SP; ++s)
      aop[p][s] = __builtin_nontemporal_load(wrow[s] + (size_t)min(k0 + p, kend - 1) * 64 + lane);

  // staging: item i of a stage is (row r, group q of 8 inputs among the stage's 64); lanes
  // walk r fastest so that the 16-byte LDS writes of a wavefront fall into distinct banks
  constexpr int ITEMS = NCT * 16 * GEMM_KS * 4;
  constexpr int IPT = (ITEMS + GEMM_THREADS - 1) / GEMM_THREADS;
  float4 xr[IPT][2];
  auto stage_load = [&](int kstage) {                     // first k-step of the stage (relative)
#pragma unroll
    for (int j = 0; j < IPT; ++j) {
      const int i = threadIdx.x + j * GEMM_THREADS;
      const int r = (i & 15) + 16 * (i / (16 * GEMM_KS * 4)), q = (i >> 4) & (GEMM_KS * 4 - 1);
      const int kk = kstage + (q >> 2);
      xr[j][0] = xr[j][1] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (i < ITEMS && m0 + r < a.M && kk < nk) {
        const float *src = a.X + (size_t)(m0 + r) * Kd + (size_t)(k0 + kk) * 32 + 8 * (q & 3);
        xr[j][0] = *reinterpret_cast<const float4 *>(src);
        xr[j][1] = *reinterpret_cast<const float4 *>(src + 4);
      }
    }
  };
  auto stage_store = [&](int buf) {
#pragma unroll
    for (int j = 0; j < IPT; ++j) {
      const int i = threadIdx.x + j * GEMM_THREADS;
      if (i < ITEMS) {
        const int r = (i & 15) + 16 * (i / (16 * GEMM_KS * 4)), q = (i >> 4) & (GEMM_KS * 4 - 1);
        const float x[8] = {xr[j][0].x, xr[j][0].y, xr[j][0].z, xr[j][0].w,
                            xr[j][1].x, xr[j][1].y, xr[j][1].z, xr[j][1].w};
        uint32_t h[4], l[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const bf16_t h0 = f32_to_bf16(x[2 * e]), h1 = f32_to_bf16(x[2 * e + 1]);
          const bf16_t l0 = f32_to_bf16(x[2 * e] - bf16_to_f32(h0));
          const bf16_t l1 = f32_to_bf16(x[2 * e + 1] - bf16_to_f32(h1));
          h[e] = (uint32_t)h0 | ((uint32_t)h1 << 16);
          l[e] = (uint32_t)l0 | ((uint32_t)l1 << 16);
        }
        const int slot = (q & 3) * 16 + (r & 15), c = r >> 4;
        bst[buf][q >> 2][2 * c][slot] = u32x4_t{h[0], h[1], h[2], h[3]};
        bst[buf][q >> 2][2 * c + 1][slot] = u32x4_t{l[0], l[1], l[2], l[3]};
      }
    }
  };

  f32x4_t acc[SP][NCT];
#pragma unroll
  for (int s = 0; s < SP; ++s)
#pragma unroll
    for (int c = 0; c < NCT; ++c) acc[s][c] = {0.f, 0.f, 0.f, 0.f};

  stage_load(0);
  stage_store(0);
  gemm_lds_barrier();

  for (int t0 = 0; t0 < nkp; t0 += GEMM_UNR) {
#pragma unroll
    for (int tu = 0; tu < GEMM_UNR; ++tu) {
      const int t = t0 + tu;                              // k-step relative to k0
      const int buf = (t0 / GEMM_KS) & 1, u = tu % GEMM_KS;
      if (u == 0) stage_load(t + GEMM_KS);                // rows of the next stage, in flight
#pragma unroll
      for (int hl = 0; hl < 2; ++hl) {
        bf16x8_t b[NCT];
#pragma unroll
        for (int c = 0; c < NCT; ++c) b[c] = __builtin_bit_cast(bf16x8_t, bst[buf][u][2 * c + hl][lane]);
#pragma unroll
        for (int s = 0; s < SP; ++s) {
          const bf16x8_t av = __builtin_bit_cast(bf16x8_t, aop[tu % GEMM_PD][s]);
#pragma unroll
          for (int c = 0; c < NCT; ++c)
            acc[s][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, b[c], acc[s][c], 0, 0, 0);
        }
      }
      // refill the ring slot just consumed (clamped: reloads of the last tile are never used)
#pragma unroll
      for (int s = 0; s < SP; ++s)
        aop[tu % GEMM_PD][s] =
            __builtin_nontemporal_load(wrow[s] + (size_t)min(k0 + t + GEMM_PD, kend - 1) * 64 + lane);
      // keep the k-steps apart: hoisting the next step's operand reads over this step's
      // products would need more registers than a wavefront has
      __builtin_amdgcn_sched_barrier(0);
      if (u == GEMM_KS - 1) {
        stage_store(buf ^ 1);
        gemm_lds_barrier();
      }
    }
  }

  // D[i][j] of a tile: output i = 4*(lane/16) + reg of the strip, row j = lane%16 of the tile
  const int j = lane & 15, i4 = (lane >> 4) * 4;
#pragma unroll
  for (int s = 0; s < SP; ++s) {
    if (s < ns) {
      const int col = (sfirst + s) * 16 + i4;
#pragma unroll
      for (int c = 0; c < NCT; ++c) {
        const int m = m0 + 16 * c + j;
        if (m < a.M) {
          const f32x4_t v = acc[s][c];
          if constexpr (EPI == 1) {
            if (col < a.n_cols) {
              const float h0 = v[0] / (1.0f + expf(-v[0])) * v[2];
              const float h1 = v[1] / (1.0f + expf(-v[1])) * v[3];
              *reinterpret_cast<float2 *>(a.out + (size_t)m * a.out_stride + (col >> 1)) =
                  make_float2(h0, h1);
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

template <int NCT, int EPI>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_bf16_kernel(GemmArgs a) {
  __shared__ u32x4_t bst[2][GEMM_KS][NCT * 2][64];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int gc_count = a.ngroups * a.nchunks;
  for (int unit = blockIdx.x; unit < a.units; unit += gridDim.x) {
    // row blocks of one (group, chunk) sit 8 units apart: same XCD, about the same time, so
    // the second reader of a weight tile finds it in that XCD's L2
    const int blk = unit / (8 * a.row_blocks), within = unit % (8 * a.row_blocks);
    const int rb = within / 8, gc = blk * 8 + within % 8;
    if (gc >= gc_count) continue;
    const int group = gc / a.nchunks, chunk = gc % a.nchunks;
    const int g0 = (int)((int64_t)a.nstrips * group / a.ngroups);
    const int g1 = (int)((int64_t)a.nstrips * (group + 1) / a.ngroups);
    const int k0 = gemm_chunk_begin(a.KT, a.nchunks, chunk);
    const int nk = gemm_chunk_begin(a.KT, a.nchunks, chunk + 1) - k0;
    const int m0 = rb * 16 * NCT;
    for (int base = g0; base < g1; base += GEMM_WAVES * GEMM_SMAX) {
      const int P = min(g1 - base, GEMM_WAVES * GEMM_SMAX);
      const int per = (P + GEMM_WAVES - 1) / GEMM_WAVES;          // strips per wavefront
      const int sfirst = min(base + wave * per, g1 - 1);
      const int ns = max(0, min(per, base + P - (base + wave * per)));
      if (per > 4) gemm_pass<NCT, 8, EPI>(a, bst, m0, chunk, k0, nk, sfirst, ns);
      else if (per > 2) gemm_pass<NCT, 4, EPI>(a, bst, m0, chunk, k0, nk, sfirst, ns);
      else if (per == 2) gemm_pass<NCT, 2, EPI>(a, bst, m0, chunk, k0, nk, sfirst, ns);
      else gemm_pass<NCT, 1, EPI>(a, bst, m0, chunk, k0, nk, sfirst, ns);
    }
  }
}

int g_gemm_wgs = 256;      // resident workgroups: one per compute unit

// k-chunks of a matrix on this path: fixed per matrix so that a row's sums do not depend on
// the call.  Matrices with few strips are cut along k until (strip ranges of >= 8 strips) x
// chunks fill the compute units; chunks are at least 16 k-steps long.
int gemm_bf16_chunks(int Kd, int nstrips) {
  const int KT = Kd / 32;
  const int groups_max = (nstrips + GEMM_WAVES - 1) / GEMM_WAVES;
  if (groups_max >= g_gemm_wgs) return 1;
  int nch = (g_gemm_wgs + groups_max / 2) / groups_max;
  nch = min(nch, max(1, KT / 16));
  return max(1, nch);
}

hipError_t launch_gemm_bf16(const DeviceMatrix &W, int strip0, int nstrips, const float *X, int M,
                            float *out, int out_stride, size_t chunk_stride, int nchunks, int epi,
                            hipStream_t st) {
  if (M < 1 || nstrips < 1 || nchunks < 1 || (epi == 1 && nchunks != 1)) return hipErrorInvalidValue;
  GemmArgs a;
  a.Wp = (const u32x4_t *)W.data;
  a.X = X;
  a.out = out;
  a.chunk_stride = chunk_stride;
  a.M = M;
  a.KT = W.Kd / 32;
  a.nchunks = nchunks;
  a.strip0 = strip0;
  a.nstrips = nstrips;
  a.n_cols = min(nstrips * 16, W.n_real - strip0 * 16);
  a.out_stride = out_stride;
  const int nct = M <= 32 ? 2 : (M <= 64 ? 4 : 8);
  a.row_blocks = (M + 16 * nct - 1) / (16 * nct);
  const int groups_max = (nstrips + GEMM_WAVES - 1) / GEMM_WAVES;
  a.ngroups = max(1, min(groups_max, g_gemm_wgs / (nchunks * a.row_blocks)));
  const int gc = a.ngroups * nchunks;
  a.units = (gc + 7) / 8 * 8 * a.row_blocks;
  const dim3 grid(min(a.units, 2 * g_gemm_wgs)), block(GEMM_THREADS);
#define DART_GEMM_GO(NCT_)                                                                   \
  do {                                                                                       \
    if (epi == 1) hipLaunchKernelGGL((gemm_bf16_kernel<NCT_, 1>), grid, block, 0, st, a);    \
    else hipLaunchKernelGGL((gemm_bf16_kernel<NCT_, 0>), grid, block, 0, st, a);             \
  } while (0)
  if (nct == 2) DART_GEMM_GO(2);
  else if (nct == 4) DART_GEMM_GO(4);
  else DART_GEMM_GO(8);
#undef DART_GEMM_GO
  return hipGetLastError();
}

}  // namespace dart
