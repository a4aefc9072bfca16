// Per-position candidate extraction (paper Alg. 1 "Top-k_i tokens from l_i" and
// s_logit = log(softmax(l)_{i,t} + eps), App. D): one read of each logit row yields the
// k best tokens and the row's log-sum-exp together.
//
// Phase 1 (grid: vocab chunks x rows): a workgroup holds a 4096-logit chunk in registers, 1024
// per wavefront.  Each wavefront computes its (max, sum exp) and extracts its k largest entries
// with wavefront-wide reductions only (no barriers); wavefront 0 then reduces the 4 x k
// candidates to the chunk's k and combines the four statistics.
// Phase 2 (grid: rows, one wavefront each): merges the chunk statistics into the row's
// log-sum-exp and extracts the k largest of the chunk winners, candidates held in registers.
// Ordering key: (logit descending, token id ascending), as one 64-bit integer
// (order-preserving float map << 32 | ~id), so extraction is a repeated integer max and the
// result is deterministic.
#include "common.h"
#include "dart_internal.h"

namespace dart {

constexpr int TOPK_THREADS = 256;
constexpr int TOPK_WAVES = TOPK_THREADS / 64;
constexpr int TOPK_PER_THREAD = 16;
constexpr int TOPK_CHUNK = TOPK_THREADS * TOPK_PER_THREAD;   // 4096
constexpr int TOPK_MERGE_REGS = 40;                          // candidates per lane in phase 2

// k repeated max-extractions over N register-resident keys per lane (0 = no key);
// emit(it, best) is called by every lane with the wavefront-wide it-th largest key.
template <int N, typename Emit>
__device__ __forceinline__ void wave_extract(const uint64_t (&key)[N], int k, Emit emit) {
  uint64_t bound = ~(uint64_t)0;
  for (int it = 0; it < k; ++it) {
    uint64_t best = 0;
#pragma unroll
    for (int e = 0; e < N; ++e)
      if (key[e] < bound && key[e] > best) best = key[e];
    best = wave_max_u64(best);
    emit(it, best);
    bound = best;            // keys are unique (they embed the token id), except the 0 filler
    if (best == 0) {
      for (int r = it + 1; r < k; ++r) emit(r, (uint64_t)0);
      break;
    }
  }
}

__global__ __launch_bounds__(TOPK_THREADS) void topk_chunk_kernel(const float *__restrict__ logits,
                                                                  int vocab, int k, int nchunks,
                                                                  uint64_t *__restrict__ cand,
                                                                  float *__restrict__ ms) {
  __shared__ uint64_t wcand[TOPK_WAVES][DART_MAX_TOPK];
  __shared__ float wms[TOPK_WAVES][2];
  const int chunk = blockIdx.x, row = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float *src = logits + (size_t)row * vocab;
  const int base = chunk * TOPK_CHUNK + wave * (TOPK_CHUNK / TOPK_WAVES);
  uint64_t key[TOPK_PER_THREAD];
  float val[TOPK_PER_THREAD];
  float mx = -3.0e38f;
#pragma unroll
  for (int e = 0; e < TOPK_PER_THREAD; ++e) {
    const int idx = base + e * 64 + lane;
    if (idx < vocab) {
      val[e] = src[idx];
      key[e] = ((uint64_t)f32_sortable(val[e]) << 32) | (uint32_t)(~(uint32_t)idx);
      mx = fmaxf(mx, val[e]);
    } else {
      val[e] = -3.0e38f;
      key[e] = 0;                                  // below every real key
    }
  }
  mx = wave_max(mx);
  float se = 0.f;
#pragma unroll
  for (int e = 0; e < TOPK_PER_THREAD; ++e)
    if (key[e] != 0) se += expf(val[e] - mx);
  se = wave_sum(se);
  if (lane == 0) {
    wms[wave][0] = mx;
    wms[wave][1] = se;
  }
  wave_extract(key, k, [&](int it, uint64_t best) {
    if (lane == 0) wcand[wave][it] = best;
  });
  __syncthreads();
  if (wave != 0) return;
  // chunk statistics in wavefront order (deterministic), then the chunk's k best of 4 x k
  const size_t slot = (size_t)row * nchunks + chunk;
  float cm = wms[0][0];
#pragma unroll
  for (int w = 1; w < TOPK_WAVES; ++w) cm = fmaxf(cm, wms[w][0]);
  float cs = 0.f;
#pragma unroll
  for (int w = 0; w < TOPK_WAVES; ++w) cs += wms[w][1] * expf(wms[w][0] - cm);
  if (lane == 0) {
    ms[slot * 2] = cm;
    ms[slot * 2 + 1] = cs;
  }
  uint64_t mine[TOPK_WAVES];
#pragma unroll
  for (int w = 0; w < TOPK_WAVES; ++w) mine[w] = lane < k ? wcand[w][lane] : 0;
  wave_extract(mine, k, [&](int it, uint64_t best) {
    if (lane == 0) cand[slot * DART_MAX_TOPK + it] = best;   // 0 when the chunk ran out
  });
}

__global__ __launch_bounds__(64) void topk_merge_kernel(const uint64_t *__restrict__ cand,
                                                        const float *__restrict__ ms, int k,
                                                        int nchunks, float eps,
                                                        int32_t *__restrict__ ids,
                                                        float *__restrict__ scores) {
  const int row = blockIdx.x, lane = threadIdx.x;
  // log-sum-exp of the row from the chunk statistics (fixed order -> deterministic)
  float mx = -3.0e38f;
  for (int c = lane; c < nchunks; c += 64) mx = fmaxf(mx, ms[((size_t)row * nchunks + c) * 2]);
  mx = wave_max(mx);
  float se = 0.f;
  for (int c = lane; c < nchunks; c += 64) {
    const size_t slot = (size_t)row * nchunks + c;
    se += ms[slot * 2 + 1] * expf(ms[slot * 2] - mx);
  }
  se = wave_sum(se);
  const float lse = mx + logf(se);
  auto emit = [&](int it, uint64_t best) {
    if (lane == 0) {
      const float logit = f32_unsortable((uint32_t)(best >> 32));
      ids[(size_t)row * k + it] = (int32_t)(~(uint32_t)best);
      scores[(size_t)row * k + it] = fminf(0.f, logf(expf(logit - lse) + eps));
    }
  };
  const int total = nchunks * k;
  const uint64_t *src = cand + (size_t)row * nchunks * DART_MAX_TOPK;
  if (total <= 64 * TOPK_MERGE_REGS) {
    uint64_t mine[TOPK_MERGE_REGS];
#pragma unroll
    for (int e = 0; e < TOPK_MERGE_REGS; ++e) {
      const int j = e * 64 + lane;
      mine[e] = j < total ? src[(size_t)(j / k) * DART_MAX_TOPK + j % k] : 0;
    }
    wave_extract(mine, k, emit);
  } else {                                          // very large vocab x k: re-read from memory
    uint64_t bound = ~(uint64_t)0;
    for (int it = 0; it < k; ++it) {
      uint64_t best = 0;
      for (int j = lane; j < total; j += 64) {
        const uint64_t key = src[(size_t)(j / k) * DART_MAX_TOPK + j % k];
        if (key < bound && key > best) best = key;
      }
      best = wave_max_u64(best);
      emit(it, best);
      bound = best;
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
  hipLaunchKernelGGL(topk_merge_kernel, dim3(rows), dim3(64), 0, st, c->topk_cand,
                     c->topk_ms, k, nchunks, eps, ids, scores);
  return hipGetLastError();
}

}  // namespace dart
