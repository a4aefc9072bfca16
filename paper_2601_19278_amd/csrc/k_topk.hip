// Per-position candidate extraction (paper Alg. 1 "Top-k_i tokens from l_i" and
// s_logit = log(softmax(l)_{i,t} + eps), App. D): one read of each logit row yields the
// k best tokens and the row's log-sum-exp together.
//
// Phase 1 (grid: vocab chunks x rows): each workgroup holds a 4096-logit chunk in
// registers, computes the chunk's (max, sum exp) and extracts its k largest entries.
// Phase 2 (grid: rows): merges the chunk statistics into the row's log-sum-exp and
// extracts the k largest of the chunk winners.
// Ordering key: (logit descending, token id ascending), as one 64-bit integer
// (order-preserving float map << 32 | ~id), so extraction is a repeated integer max and the
// result is deterministic.
#include "common.h"
#include "dart_internal.h"

namespace dart {

constexpr int TOPK_THREADS = 256;
constexpr int TOPK_PER_THREAD = 16;
constexpr int TOPK_CHUNK = TOPK_THREADS * TOPK_PER_THREAD;   // 4096

__device__ __forceinline__ uint64_t block_max_u64(uint64_t v, uint64_t *red) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  v = wave_max_u64(v);
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  uint64_t t = red[0];
  for (int w = 1; w < TOPK_THREADS / 64; ++w) t = red[w] > t ? red[w] : t;
  return t;
}

__global__ __launch_bounds__(TOPK_THREADS) void topk_chunk_kernel(const float *__restrict__ logits,
                                                                  int vocab, int k, int nchunks,
                                                                  uint64_t *__restrict__ cand,
                                                                  float *__restrict__ ms) {
  __shared__ float red[16];
  __shared__ uint64_t red64[4];
  const int chunk = blockIdx.x, row = blockIdx.y, t = threadIdx.x;
  const float *src = logits + (size_t)row * vocab;
  const int base = chunk * TOPK_CHUNK;
  uint64_t key[TOPK_PER_THREAD];
  float val[TOPK_PER_THREAD];
  float mx = -3.0e38f;
#pragma unroll
  for (int e = 0; e < TOPK_PER_THREAD; ++e) {
    const int idx = base + e * TOPK_THREADS + t;
    if (idx < vocab) {
      val[e] = src[idx];
      key[e] = ((uint64_t)f32_sortable(val[e]) << 32) | (uint32_t)(~(uint32_t)idx);
      mx = fmaxf(mx, val[e]);
    } else {
      val[e] = -3.0e38f;
      key[e] = 0;                                  // below every real key
    }
  }
  mx = block_max(mx, red);
  float se = 0.f;
#pragma unroll
  for (int e = 0; e < TOPK_PER_THREAD; ++e)
    if (key[e] != 0) se += expf(val[e] - mx);
  se = block_sum(se, red);
  const size_t slot = (size_t)row * nchunks + chunk;
  if (t == 0) {
    ms[slot * 2] = mx;
    ms[slot * 2 + 1] = se;
  }
  uint64_t bound = ~(uint64_t)0;
  for (int it = 0; it < k; ++it) {
    uint64_t best = 0;
#pragma unroll
    for (int e = 0; e < TOPK_PER_THREAD; ++e)
      if (key[e] < bound && key[e] > best) best = key[e];
    best = block_max_u64(best, red64);
    if (t == 0) cand[slot * DART_MAX_TOPK + it] = best;   // 0 when the chunk ran out
    bound = best;
    if (best == 0) {                                      // uniform: fill the rest and stop
      for (int r = it + 1 + t; r < k; r += TOPK_THREADS) cand[slot * DART_MAX_TOPK + r] = 0;
      break;
    }
  }
}

__global__ __launch_bounds__(TOPK_THREADS) void topk_merge_kernel(
    const uint64_t *__restrict__ cand, const float *__restrict__ ms, int k, int nchunks, float eps,
    int32_t *__restrict__ ids, float *__restrict__ scores) {
  __shared__ float red[16];
  __shared__ uint64_t red64[4];
  const int row = blockIdx.x, t = threadIdx.x;
  // log-sum-exp of the row from the chunk statistics (fixed order -> deterministic)
  float mx = -3.0e38f;
  for (int c = t; c < nchunks; c += TOPK_THREADS) mx = fmaxf(mx, ms[((size_t)row * nchunks + c) * 2]);
  mx = block_max(mx, red);
  float se = 0.f;
  for (int c = t; c < nchunks; c += TOPK_THREADS) {
    const size_t slot = (size_t)row * nchunks + c;
    se += ms[slot * 2 + 1] * expf(ms[slot * 2] - mx);
  }
  se = block_sum(se, red);
  const float lse = mx + logf(se);

  const int total = nchunks * k;
  uint64_t bound = ~(uint64_t)0;
  for (int it = 0; it < k; ++it) {
    uint64_t best = 0;
    for (int j = t; j < total; j += TOPK_THREADS) {
      const uint64_t key = cand[((size_t)row * nchunks + j / k) * DART_MAX_TOPK + j % k];
      if (key < bound && key > best) best = key;
    }
    best = block_max_u64(best, red64);
    bound = best;
    if (t == 0) {
      const float logit = f32_unsortable((uint32_t)(best >> 32));
      ids[(size_t)row * k + it] = (int32_t)(~(uint32_t)best);
      scores[(size_t)row * k + it] = fminf(0.f, logf(expf(logit - lse) + eps));
    }
  }
}

hipError_t launch_topk(const dart_ctx *c, const float *logits, int rows, int vocab, int k, float eps,
                       int32_t *ids, float *scores, hipStream_t st) {
  const int nchunks = (vocab + TOPK_CHUNK - 1) / TOPK_CHUNK;
  hipLaunchKernelGGL(topk_chunk_kernel, dim3(nchunks, rows), dim3(TOPK_THREADS), 0, st, logits,
                     vocab, k, nchunks, c->topk_cand, c->topk_ms);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(topk_merge_kernel, dim3(rows), dim3(TOPK_THREADS), 0, st, c->topk_cand,
                     c->topk_ms, k, nchunks, eps, ids, scores);
  return hipGetLastError();
}

}  // namespace dart
