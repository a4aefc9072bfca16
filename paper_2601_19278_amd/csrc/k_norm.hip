// Row-wise kernels of the draft layer: input gather + RMSNorm, residual + RMSNorm, SwiGLU.
// (Draft layer = one pre-norm decoder layer, paper Sec. 3.2 / App. B.)
#include "common.h"
#include "dart_internal.h"

namespace dart {

constexpr int ROW_THREADS = 512;
constexpr int ROW_MAXIT = 4;            // 8 * ROW_THREADS * ROW_MAXIT = 16384 features at most

// Eight consecutive elements of a row as floats (one 16- or 32-byte access).
__device__ __forceinline__ void load8(const float *p, float *v) {
  const float4 a = *reinterpret_cast<const float4 *>(p), b = *reinterpret_cast<const float4 *>(p + 4);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void load8(const bf16_t *p, float *v) {
  const uint4 a = *reinterpret_cast<const uint4 *>(p);
  const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    v[2 * i] = __uint_as_float(w[i] << 16);
    v[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
  }
}
__device__ __forceinline__ void store8(float *p, const float *v) {
  *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
  *reinterpret_cast<float4 *>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}

// Row r of the pass is position pos of sequence b of [z_1..z_n, MASK x (K-1)] (Sec. 3.2): a
// prefix row of that sequence's `hidden` when pos < n, else mask embedding pos-n.  Writes the
// RMS-normed row (times gain) to xn[r] and, for query rows, the raw row to resid[b*K + j].
// One workgroup per row; the row stays in registers between the two passes, and all loads
// of a pass are issued before the first use (the kernel is pure latency otherwise).
// pack != null: the normed rows are written as the packed operand tiles of the multi-row
// projection that consumes them instead of xn (see resid_norm_kernel).
template <typename T>
__global__ __launch_bounds__(ROW_THREADS) void rmsnorm_gather_kernel(
    SeqBatch sb, const T *__restrict__ mask_emb, const T *__restrict__ gain, int d, float eps,
    float *__restrict__ xn, float *__restrict__ resid, uint4 *__restrict__ pack, int ntiles,
    int ksteps, int terms) {
  __shared__ float red[16];
  const int i = blockIdx.x;
  if (i >= sb.row_off[sb.B]) {              // padding rows of the packed operand (uniform)
    for (int c = threadIdx.x * 8; c < ksteps * 32; c += ROW_THREADS * 8) pack_zero8(pack, ntiles, terms, i, c);
    return;
  }
  if (pack)
    for (int c = d + threadIdx.x * 8; c < ksteps * 32; c += ROW_THREADS * 8) pack_zero8(pack, ntiles, terms, i, c);
  int b, pos, qi;
  seq_of_row(sb, i, b, pos, qi);
  const int n = sb.n[b];
  const T *src = pos < n ? (const T *)sb.hidden[b] + (size_t)pos * d
                         : mask_emb + (size_t)(pos - n) * d;
  float v[ROW_MAXIT][8], g[ROW_MAXIT][8];
#pragma unroll
  for (int j = 0; j < ROW_MAXIT; ++j) {
    const int c = (j * ROW_THREADS + threadIdx.x) * 8;
    if (c < d) {
      load8(src + c, v[j]);
      load8(gain + c, g[j]);
    }
  }
  float ss = 0.f;
#pragma unroll
  for (int j = 0; j < ROW_MAXIT; ++j)
    if ((j * ROW_THREADS + threadIdx.x) * 8 < d)
#pragma unroll
      for (int e = 0; e < 8; ++e) ss += v[j][e] * v[j][e];
  ss = block_sum(ss, red);
  const float rstd = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
  for (int j = 0; j < ROW_MAXIT; ++j) {
    const int c = (j * ROW_THREADS + threadIdx.x) * 8;
    if (c < d) {
      if (qi >= 0) store8(resid + (size_t)(b * sb.K + qi) * d + c, v[j]);
#pragma unroll
      for (int e = 0; e < 8; ++e) v[j][e] = v[j][e] * rstd * g[j][e];
      if (pack)
        pack_store8(pack, ntiles, terms, i, c, v[j]);
      else
        store8(xn + (size_t)i * d + c, v[j]);
    }
  }
}

// The input norm of many rows (the K/V build of a long prefix) in two steps, so that the packed
// operand tiles are written as whole 1 KiB tiles: row_rstd_kernel computes 1/rms of every pass
// row exactly as rmsnorm_gather_kernel does (same thread-to-column map, same reduction order:
// the two must agree bit for bit, since rows normed by either end up in one K/V buffer), and
// pack_norm_tiles_kernel forms (x * rstd) * gain per element -- again the same arithmetic -- and
// writes the two-term tiles, one tile pair per wavefront store.
template <typename T>
__global__ __launch_bounds__(ROW_THREADS) void row_rstd_kernel(SeqBatch sb, const T *__restrict__ mask_emb,
                                                              int d, float eps, float *__restrict__ rstd) {
  __shared__ float red[16];
  const int i = blockIdx.x;
  int b, pos, qi;
  seq_of_row(sb, i, b, pos, qi);
  const int n = sb.n[b];
  const T *src = pos < n ? (const T *)sb.hidden[b] + (size_t)pos * d : mask_emb + (size_t)(pos - n) * d;
  float v[ROW_MAXIT][8];
#pragma unroll
  for (int j = 0; j < ROW_MAXIT; ++j) {
    const int c = (j * ROW_THREADS + threadIdx.x) * 8;
    if (c < d) load8(src + c, v[j]);
  }
  float ss = 0.f;
#pragma unroll
  for (int j = 0; j < ROW_MAXIT; ++j)
    if ((j * ROW_THREADS + threadIdx.x) * 8 < d)
#pragma unroll
      for (int e = 0; e < 8; ++e) ss += v[j][e] * v[j][e];
  ss = block_sum(ss, red);
  if (threadIdx.x == 0) rstd[i] = 1.0f / sqrtf(ss / (float)d + eps);
}

// grid (row tiles, ceil(k-steps / 16)), 8 wavefronts, each two adjacent k-steps of its row tile:
// lane (gq, col) owns inputs 32 t + 8 gq .. + 7 of row 16 tile + col, the lane's 16 bytes of the
// hi tile and of the lo tile.  Rows beyond the pass and k-steps beyond d are written as zeros.
template <typename T>
__global__ __launch_bounds__(ROW_THREADS) void pack_norm_tiles_kernel(
    SeqBatch sb, const T *__restrict__ mask_emb, const T *__restrict__ gain,
    const float *__restrict__ rstd, int d, int ntiles, int ksteps, uint4 *__restrict__ pack) {
  const int tile = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = tile * 16 + (lane & 15), gq = lane >> 4;
  const bool row_ok = r < sb.row_off[sb.B];
  const T *src = nullptr;
  float rs = 0.f;
  if (row_ok) {
    int b, pos, qi;
    seq_of_row(sb, r, b, pos, qi);
    const int n = sb.n[b];
    src = pos < n ? (const T *)sb.hidden[b] + (size_t)pos * d : mask_emb + (size_t)(pos - n) * d;
    rs = rstd[r];
  }
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int t = (blockIdx.y * 8 + wave) * 2 + u;
    if (t >= ksteps) continue;
    const int c = t * 32 + 8 * gq;
    uint4 *dst = pack + ((size_t)t * ntiles + tile) * 128 + lane;      // two-term format
    if (row_ok && c < d) {
      float v[8], g[8];
      load8(src + c, v);
      load8(gain + c, g);
      uint32_t h[4], l[4];
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = v[e] * rs * g[e];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bf16_t h0 = f32_to_bf16(v[2 * e]), h1 = f32_to_bf16(v[2 * e + 1]);
        const bf16_t l0 = f32_to_bf16(v[2 * e] - bf16_to_f32(h0));
        const bf16_t l1 = f32_to_bf16(v[2 * e + 1] - bf16_to_f32(h1));
        h[e] = (uint32_t)h0 | ((uint32_t)h1 << 16);
        l[e] = (uint32_t)l0 | ((uint32_t)l1 << 16);
      }
      dst[0] = make_uint4(h[0], h[1], h[2], h[3]);
      dst[64] = make_uint4(l[0], l[1], l[2], l[3]);
    } else {
      dst[0] = make_uint4(0, 0, 0, 0);
      dst[64] = make_uint4(0, 0, 0, 0);
    }
  }
}

// Front end (Sec. 3.2): the concatenated target hidden states of the pass rows as fp32, the
// input format of the FC projection.  Mask rows have no features: zeros (their FC output is
// not used).  One workgroup per row.
template <typename T>
__global__ __launch_bounds__(ROW_THREADS) void feature_rows_kernel(SeqBatch sb, int feat_dim,
                                                                   float *__restrict__ out) {
  const int i = blockIdx.x;
  int b, pos, qi;
  seq_of_row(sb, i, b, pos, qi);
  const bool prefix = pos < sb.n[b];
  const T *src = (const T *)sb.hidden[b] + (size_t)(prefix ? pos : 0) * feat_dim;
  for (int c = threadIdx.x * 8; c < feat_dim; c += ROW_THREADS * 8) {
    float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (prefix) load8(src + c, v);
    store8(out + (size_t)i * feat_dim + c, v);
  }
}

// Front end (Sec. 3.2): z = [g ; e] of a pass row -- g = FC output (sum of the projection's
// k-chunk partials, in index order), e = embedding of the token that follows the position
// (shifted embeddings); a mask row takes both halves from its 2d-wide mask slot.  Each half
// gets its own RMSNorm; xn[r] = [norm(g) * gain_g ; norm(e) * gain_e], and the g half is the
// layer's residual stream (written for query rows).  One workgroup per row.
template <typename T>
__global__ __launch_bounds__(ROW_THREADS) void front_norm_kernel(
    SeqBatch sb, const float *__restrict__ fc_part, int chunks, size_t chunk_stride,
    const T *__restrict__ embed, const T *__restrict__ mask_emb, const T *__restrict__ gain_g,
    const T *__restrict__ gain_e, int d, float eps, float *__restrict__ xn,
    float *__restrict__ resid) {
  __shared__ float red[16];
  const int i = blockIdx.x;
  int b, pos, qi;
  seq_of_row(sb, i, b, pos, qi);
  const int n = sb.n[b];
  const bool prefix = pos < n;
  const T *mrow = mask_emb + (size_t)(prefix ? 0 : pos - n) * 2 * d;
  const T *erow = prefix ? embed + (size_t)sb.tokens[b][pos] * d : mrow + d;
  float g[ROW_MAXIT][8], e[ROW_MAXIT][8];
  float sg = 0.f, se = 0.f;
#pragma unroll
  for (int j = 0; j < ROW_MAXIT; ++j) {
    const int c = (j * ROW_THREADS + threadIdx.x) * 8;
    if (c < d) {
      if (prefix) {
#pragma unroll
        for (int q = 0; q < 8; ++q) g[j][q] = 0.f;
        for (int k = 0; k < chunks; ++k) {
          float p[8];
          load8(fc_part + k * chunk_stride + (size_t)i * d + c, p);
#pragma unroll
          for (int q = 0; q < 8; ++q) g[j][q] += p[q];
        }
      } else {
        load8(mrow + c, g[j]);
      }
      load8(erow + c, e[j]);
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        sg += g[j][q] * g[j][q];
        se += e[j][q] * e[j][q];
      }
    }
  }
  sg = block_sum(sg, red);
  se = block_sum(se, red);
  const float rg = 1.0f / sqrtf(sg / (float)d + eps), re = 1.0f / sqrtf(se / (float)d + eps);
#pragma unroll
  for (int j = 0; j < ROW_MAXIT; ++j) {
    const int c = (j * ROW_THREADS + threadIdx.x) * 8;
    if (c < d) {
      float wg[8], we[8];
      load8(gain_g + c, wg);
      load8(gain_e + c, we);
      if (qi >= 0) store8(resid + (size_t)(b * sb.K + qi) * d + c, g[j]);
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        g[j][q] = g[j][q] * rg * wg[q];
        e[j][q] = e[j][q] * re * we[q];
      }
      store8(xn + (size_t)i * 2 * d + c, g[j]);
      store8(xn + (size_t)i * 2 * d + d + c, e[j]);
    }
  }
}

// y = resid + sum_c part[c];  yn = RMSNorm(y) * gain.  part[c] row r starts at
// part + c*chunk_stride + r*row_stride.  Chunk partials are added in index order.
// y, yn: either may be null (not stored).
// pack != null: yn is also written as the packed operand tiles of the multi-row projection
// that consumes it (ntiles row tiles, ksteps k-steps); the grid then covers the padded rows
// ntiles*16, and rows >= rows and inputs >= d are written as zeros.
// NJ: column groups of 8 per thread (ceil(d / (8 * ROW_THREADS))).
template <typename T, int NJ>
__global__ __launch_bounds__(ROW_THREADS) void resid_norm_kernel(
    const float *__restrict__ resid, const float *__restrict__ part, int chunks, size_t chunk_stride,
    int row_stride, const T *__restrict__ gain, int rows, int d, float eps, float *__restrict__ y,
    float *__restrict__ yn, uint4 *__restrict__ pack, int ntiles, int ksteps, int terms) {
  __shared__ float red[16];
  const int r = blockIdx.x;
  if (r >= rows) {                          // padding rows of the packed operand (uniform)
    for (int c = threadIdx.x * 8; c < ksteps * 32; c += ROW_THREADS * 8) pack_zero8(pack, ntiles, terms, r, c);
    return;
  }
  if (pack)
    for (int c = d + threadIdx.x * 8; c < ksteps * 32; c += ROW_THREADS * 8) pack_zero8(pack, ntiles, terms, r, c);
  float v[NJ][8], g[NJ][8];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int c = (j * ROW_THREADS + threadIdx.x) * 8;
    if (c < d) {
      load8(resid + (size_t)r * d + c, v[j]);
      load8(gain + c, g[j]);
    }
  }
  // chunk partials, added in index order.  The loads of a batch of chunks are issued for all
  // of the thread's column groups before the first add: the kernel is one workgroup per row
  // and its time is the number of such round trips.
  constexpr int U = NJ <= 2 ? 9 : 4;     // 9: the 17 chunks of a 17408-input projection in two batches
  for (int k0 = 0; k0 < chunks; k0 += U) {
    float p[NJ][U][8];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int c = (j * ROW_THREADS + threadIdx.x) * 8;
      if (c < d) {
#pragma unroll
        for (int u = 0; u < U; ++u)
          if (k0 + u < chunks)
            load8(part + (size_t)(k0 + u) * chunk_stride + (size_t)r * row_stride + c, p[j][u]);
      }
    }
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int c = (j * ROW_THREADS + threadIdx.x) * 8;
      if (c < d) {
#pragma unroll
        for (int u = 0; u < U; ++u)
          if (k0 + u < chunks)
#pragma unroll
            for (int e = 0; e < 8; ++e) v[j][e] += p[j][u][e];
      }
    }
  }
  float ss = 0.f;
#pragma unroll
  for (int j = 0; j < NJ; ++j)
    if ((j * ROW_THREADS + threadIdx.x) * 8 < d)
#pragma unroll
      for (int e = 0; e < 8; ++e) ss += v[j][e] * v[j][e];
  ss = block_sum(ss, red);
  const float rstd = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int c = (j * ROW_THREADS + threadIdx.x) * 8;
    if (c < d) {
      if (y) store8(y + (size_t)r * d + c, v[j]);
#pragma unroll
      for (int e = 0; e < 8; ++e) v[j][e] = v[j][e] * rstd * g[j][e];
      if (yn) store8(yn + (size_t)r * d + c, v[j]);
      if (pack) pack_store8(pack, ntiles, terms, r, c, v[j]);
    }
  }
}

// h[r][f] = silu(gate) * up from the fused gate/up projection (summed over k-chunks).
// interleaved = 0: row r is [gate(ffn) | up(ffn)].
// interleaved = 1: features come in groups of 4 outputs (g f, g f+1, u f, u f+1), the row
// order the packed bf16 matrix uses so that one MFMA lane holds a gate/up pair.
__global__ __launch_bounds__(256) void swiglu_kernel(const float *__restrict__ gu, int chunks,
                                                     size_t chunk_stride, int ffn, int interleaved,
                                                     float *__restrict__ h) {
  const int r = blockIdx.y;
  const int f = blockIdx.x * blockDim.x + threadIdx.x;
  if (f >= ffn) return;
  size_t gi, ui;
  if (interleaved) {
    gi = (size_t)(f >> 1) * 4 + (f & 1);
    ui = gi + 2;
  } else {
    gi = f;
    ui = (size_t)ffn + f;
  }
  const float *row = gu + (size_t)r * 2 * ffn;
  float g = 0.f, u = 0.f;
  for (int k = 0; k < chunks; ++k) {
    g += row[k * chunk_stride + gi];
    u += row[k * chunk_stride + ui];
  }
  h[(size_t)r * ffn + f] = g / (1.0f + expf(-g)) * u;
}

// out[r][j] = sum_c part[c][r][j] (chunk partials of a projection, added in index order).
__global__ __launch_bounds__(256) void sum_chunks_kernel(const float *__restrict__ part, int chunks,
                                                         size_t chunk_stride, int row_stride, int n,
                                                         float *__restrict__ out, int out_stride) {
  const int r = blockIdx.y;
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= n) return;
  float v = 0.f;
  for (int c = 0; c < chunks; ++c) v += part[c * chunk_stride + (size_t)r * row_stride + j];
  out[(size_t)r * out_stride + j] = v;
}

hipError_t launch_sum_chunks(const float *part, int chunks, size_t chunk_stride, int row_stride,
                             int rows, int n, float *out, int out_stride, hipStream_t st) {
  hipLaunchKernelGGL(sum_chunks_kernel, dim3((n + 255) / 256, rows), dim3(256), 0, st, part, chunks,
                     chunk_stride, row_stride, n, out, out_stride);
  return hipGetLastError();
}

void gemm_bf16_pack_shape(int M, int Kd, int *ntiles, int *ksteps);

hipError_t launch_rmsnorm_gather(int dtype, const SeqBatch &sb, const void *mask_emb,
                                 const void *gain, int d, float eps, float *xn, float *resid,
                                 void *pack, int terms, hipStream_t st) {
  const int M = sb.row_off[sb.B];
  int ntiles = 0, ksteps = 0, grid = M;
  if (pack) {
    if (dtype != DART_BF16 || (d & 7)) return hipErrorInvalidValue;
    gemm_bf16_pack_shape(M, d, &ntiles, &ksteps);
    grid = ntiles * 16;
  }
  if (dtype == DART_BF16)
    hipLaunchKernelGGL(rmsnorm_gather_kernel<bf16_t>, dim3(grid), dim3(ROW_THREADS), 0, st, sb,
                       (const bf16_t *)mask_emb, (const bf16_t *)gain, d, eps, xn, resid,
                       (uint4 *)pack, ntiles, ksteps, terms);
  else
    hipLaunchKernelGGL(rmsnorm_gather_kernel<float>, dim3(grid), dim3(ROW_THREADS), 0, st, sb,
                       (const float *)mask_emb, (const float *)gain, d, eps, xn, resid,
                       (uint4 *)nullptr, 0, 0, 2);
  return hipGetLastError();
}

// Normed rows of a K/V-only pass as two-term operand tiles (bf16 storage only); rstd: scratch of
// one float per pass row.
hipError_t launch_norm_pack_rows(const SeqBatch &sb, const void *mask_emb, const void *gain, int d,
                                 float eps, float *rstd, void *pack, hipStream_t st) {
  const int M = sb.row_off[sb.B];
  if ((d & 7) || d > 8 * ROW_THREADS * ROW_MAXIT) return hipErrorInvalidValue;
  int ntiles = 0, ksteps = 0;
  gemm_bf16_pack_shape(M, d, &ntiles, &ksteps);
  hipLaunchKernelGGL(row_rstd_kernel<bf16_t>, dim3(M), dim3(ROW_THREADS), 0, st, sb,
                     (const bf16_t *)mask_emb, d, eps, rstd);
  hipLaunchKernelGGL(pack_norm_tiles_kernel<bf16_t>, dim3(ntiles, (ksteps + 15) / 16), dim3(ROW_THREADS), 0,
                     st, sb, (const bf16_t *)mask_emb, (const bf16_t *)gain, rstd, d, ntiles, ksteps,
                     (uint4 *)pack);
  return hipGetLastError();
}

hipError_t launch_feature_rows(int dtype, const SeqBatch &sb, int feat_dim, float *out, hipStream_t st) {
  const int M = sb.row_off[sb.B];
  if (dtype == DART_BF16)
    hipLaunchKernelGGL(feature_rows_kernel<bf16_t>, dim3(M), dim3(ROW_THREADS), 0, st, sb, feat_dim, out);
  else
    hipLaunchKernelGGL(feature_rows_kernel<float>, dim3(M), dim3(ROW_THREADS), 0, st, sb, feat_dim, out);
  return hipGetLastError();
}

hipError_t launch_front_norm(int dtype, const SeqBatch &sb, const float *fc_part, int chunks,
                             size_t chunk_stride, const void *embed, const void *mask_emb,
                             const void *gain_g, const void *gain_e, int d, float eps, float *xn,
                             float *resid, hipStream_t st) {
  const int M = sb.row_off[sb.B];
  if (dtype == DART_BF16)
    hipLaunchKernelGGL(front_norm_kernel<bf16_t>, dim3(M), dim3(ROW_THREADS), 0, st, sb, fc_part,
                       chunks, chunk_stride, (const bf16_t *)embed, (const bf16_t *)mask_emb,
                       (const bf16_t *)gain_g, (const bf16_t *)gain_e, d, eps, xn, resid);
  else
    hipLaunchKernelGGL(front_norm_kernel<float>, dim3(M), dim3(ROW_THREADS), 0, st, sb, fc_part,
                       chunks, chunk_stride, (const float *)embed, (const float *)mask_emb,
                       (const float *)gain_g, (const float *)gain_e, d, eps, xn, resid);
  return hipGetLastError();
}

hipError_t launch_resid_norm(int dtype, const float *resid, const float *part, int chunks,
                             size_t chunk_stride, int row_stride, const void *gain, int rows, int d,
                             float eps, float *y, float *yn, void *pack, int terms, hipStream_t st) {
  int ntiles = 0, ksteps = 0, grid = rows;
  if (pack) {
    if (dtype != DART_BF16 || (d & 7)) return hipErrorInvalidValue;
    gemm_bf16_pack_shape(rows, d, &ntiles, &ksteps);
    grid = ntiles * 16;
  }
  const int nj = (d + 8 * ROW_THREADS - 1) / (8 * ROW_THREADS);
  if (nj > ROW_MAXIT) return hipErrorInvalidValue;
#define DART_RESID_NORM_GO(NJ_)                                                                     \
  do {                                                                                              \
    if (dtype == DART_BF16)                                                                         \
      hipLaunchKernelGGL((resid_norm_kernel<bf16_t, NJ_>), dim3(grid), dim3(ROW_THREADS), 0, st,    \
                         resid, part, chunks, chunk_stride, row_stride, (const bf16_t *)gain, rows, \
                         d, eps, y, yn, (uint4 *)pack, ntiles, ksteps, terms);                      \
    else                                                                                            \
      hipLaunchKernelGGL((resid_norm_kernel<float, NJ_>), dim3(grid), dim3(ROW_THREADS), 0, st,     \
                         resid, part, chunks, chunk_stride, row_stride, (const float *)gain, rows,  \
                         d, eps, y, yn, (uint4 *)nullptr, 0, 0, 2);                                 \
  } while (0)
  if (nj == 1) DART_RESID_NORM_GO(1);
  else if (nj == 2) DART_RESID_NORM_GO(2);
  else DART_RESID_NORM_GO(4);
#undef DART_RESID_NORM_GO
  return hipGetLastError();
}

hipError_t launch_swiglu(const float *gu, int chunks, size_t chunk_stride, int rows, int ffn,
                         int interleaved, float *h, hipStream_t st) {
  hipLaunchKernelGGL(swiglu_kernel, dim3((ffn + 255) / 256, rows), dim3(256), 0, st, gu, chunks,
                     chunk_stride, ffn, interleaved, h);
  return hipGetLastError();
}

}  // namespace dart
