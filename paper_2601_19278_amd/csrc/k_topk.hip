// Per-position candidate extraction (paper Alg. 1 "Top-k_i tokens from l_i" and
// s_logit = log(softmax(l)_{i,t} + eps), App. D): one read of each logit row yields the
// k best tokens and the row's log-sum-exp together, in one launch.
//
// Grid: vocab chunks x rows.  A workgroup holds a 4096-logit chunk in registers, 1024 per
// wavefront.  Each wavefront computes its (max, sum exp) and selects its k largest entries;
// wavefront 0 then reduces the 4 x k winners to the chunk's k, combines the four statistics
// and publishes both.  The workgroup that publishes a row's last chunk (a counter per row,
// reset by that same workgroup) merges the chunk statistics into the row's log-sum-exp and
// selects the k largest of the chunk winners: no second launch, and the result does not
// depend on which workgroup happens to be last.
//
// Selection inside a wavefront (wave_select): the k-th largest of the 64 lane maxima is a
// lower bound T of the k-th largest value, found (to 16 bits) by a bitwise search with ballots;
// the entries >= T (at least k, in practice few more) are compacted into LDS and ranked by
// counting.  This replaces k dependent wavefront-wide max reductions by a handful of
// independent steps.  If ties make the candidate set overflow its LDS buffer the code falls
// back to the k sequential extractions.
// Ordering key: (logit descending, token id ascending), as one 64-bit integer
// (order-preserving float map << 32 | ~id), unique per entry, so the result is deterministic.
#include "common.h"
#include "dart_internal.h"

namespace dart {

constexpr int TOPK_THREADS = 256;
constexpr int TOPK_WAVES = TOPK_THREADS / 64;
constexpr int TOPK_PER_THREAD = 16;
constexpr int TOPK_CHUNK = TOPK_THREADS * TOPK_PER_THREAD;   // 4096
constexpr int TOPK_MERGE_REGS = 40;                          // candidates per lane in the merge
constexpr int TOPK_CAP = 256;                                // compacted candidates per selection

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

// The k largest of the wavefront's 64 x N keys (0 = no key), in descending order:
// emit(rank, key) is called once per rank < k by some lane (key 0 when fewer than k exist).
// buf: TOPK_CAP keys of LDS owned by this wavefront.  Must be called by all 64 lanes.
template <int N, typename Emit>
__device__ __forceinline__ void wave_select(const uint64_t (&key)[N], int k, uint64_t *buf, Emit emit) {
  const int lane = threadIdx.x & 63;
  uint32_t hm = 0;                       // lane maximum of the value words (real keys are > 0)
#pragma unroll
  for (int e = 0; e < N; ++e) hm = max(hm, (uint32_t)(key[e] >> 32));
  // T: at least k lane maxima are >= T.  Searched bit by bit from the top and only down to bit
  // 16 (sign, exponent and 7 significand bits): the low bits would only trim the few entries
  // that share that prefix with the k-th lane maximum, and each step is a dependent
  // compare-ballot-count round trip.
  uint32_t T = 0;
  for (int bit = 31; bit >= 16; --bit) {
    const uint32_t trial = T | (1u << bit);
    if (__popcll(__ballot(hm >= trial)) >= k) T = trial;
  }
  int c = 0;
#pragma unroll
  for (int e = 0; e < N; ++e) c += key[e] != 0 && (uint32_t)(key[e] >> 32) >= T;
  const int incl = wave_scan_add_dpp(c);  // inclusive prefix sum over the lanes
  const int m = __builtin_amdgcn_readlane(incl, 63);
  if (m > TOPK_CAP) {                    // heavy ties: sequential extraction
    wave_extract(key, k, [&](int it, uint64_t best) {
      if (lane == 0) emit(it, best);
    });
    return;
  }
  int at = incl - c;
#pragma unroll
  for (int e = 0; e < N; ++e)
    if (key[e] != 0 && (uint32_t)(key[e] >> 32) >= T) buf[at++] = key[e];
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  for (int i = lane; i < m; i += 64) {
    const uint64_t mine = buf[i];
    int r = 0;
#pragma unroll 4
    for (int j = 0; j < m; ++j) r += buf[j] > mine;
    if (r < k) emit(r, mine);
  }
  for (int r = m + lane; r < k; r += 64) emit(r, (uint64_t)0);
}

// Results that another workgroup (possibly on another XCD, behind another L2) reads in the same
// launch are written and read with device-scope accesses: they go to the point of coherence
// without a cache-wide write-back or invalidate, which a __threadfence() per workgroup would
// cost.  Order: a publisher waits until its stores are acknowledged, then bumps the row's
// counter; the workgroup that reads the final count issues its loads after that read.
template <typename T>
__device__ __forceinline__ void publish(T *p, T v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T>
__device__ __forceinline__ T fetch(const T *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ __launch_bounds__(TOPK_THREADS) void topk_kernel(
    const float *__restrict__ logits, int vocab, int k, int nchunks, float eps,
    uint64_t *cand, float *ms, int32_t *row_count,
    int32_t *__restrict__ ids, float *__restrict__ scores) {
  __shared__ uint64_t wcand[TOPK_WAVES][DART_MAX_TOPK];
  __shared__ uint64_t sel[TOPK_WAVES][TOPK_CAP];
  __shared__ float wms[TOPK_WAVES][2];
  __shared__ int is_last;
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
  mx = wave_max_dpp(mx);
  float se = 0.f;
#pragma unroll
  for (int e = 0; e < TOPK_PER_THREAD; ++e)
    if (key[e] != 0) se += expf(val[e] - mx);
  se = wave_sum_dpp(se);
  if (lane == 0) {
    wms[wave][0] = mx;
    wms[wave][1] = se;
  }
  wave_select(key, k, sel[wave], [&](int r, uint64_t best) { wcand[wave][r] = best; });
  __syncthreads();
  const size_t slot = (size_t)row * nchunks + chunk;
  if (wave == 0) {
    // chunk statistics in wavefront order (deterministic), then the chunk's k best of 4 x k
    float cm = wms[0][0];
#pragma unroll
    for (int w = 1; w < TOPK_WAVES; ++w) cm = fmaxf(cm, wms[w][0]);
    float cs = 0.f;
#pragma unroll
    for (int w = 0; w < TOPK_WAVES; ++w) cs += wms[w][1] * expf(wms[w][0] - cm);
    if (lane == 0) {
      publish(&ms[slot * 2], cm);
      publish(&ms[slot * 2 + 1], cs);
    }
    uint64_t mine[TOPK_WAVES];
#pragma unroll
    for (int w = 0; w < TOPK_WAVES; ++w) mine[w] = lane < k ? wcand[w][lane] : 0;
    wave_select(mine, k, sel[0], [&](int r, uint64_t best) {
      publish(&cand[slot * DART_MAX_TOPK + r], best);       // 0 when the chunk ran out
    });
    // results first (all lanes' stores acknowledged), then the row's arrival count
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (lane == 0)
      is_last = __hip_atomic_fetch_add(&row_count[row], 1, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT) == nchunks - 1;
  }
  __syncthreads();
  if (!is_last || wave != 0) return;
  if (lane == 0) publish(&row_count[row], 0);      // ready for the next call

  // the row's last chunk is in: log-sum-exp from the chunk statistics (fixed order)
  float rmx = -3.0e38f;
  for (int c = lane; c < nchunks; c += 64) rmx = fmaxf(rmx, fetch(&ms[((size_t)row * nchunks + c) * 2]));
  rmx = wave_max_dpp(rmx);
  float rse = 0.f;
  for (int c = lane; c < nchunks; c += 64) {
    const size_t sl = (size_t)row * nchunks + c;
    rse += fetch(&ms[sl * 2 + 1]) * expf(fetch(&ms[sl * 2]) - rmx);
  }
  rse = wave_sum_dpp(rse);
  const float lse = rmx + logf(rse);
  auto emit = [&](int it, uint64_t best) {
    const float logit = f32_unsortable((uint32_t)(best >> 32));
    ids[(size_t)row * k + it] = (int32_t)(~(uint32_t)best);
    scores[(size_t)row * k + it] = fminf(0.f, logf(expf(logit - lse) + eps));
  };
  const int total = nchunks * k;
  const uint64_t *csrc = cand + (size_t)row * nchunks * DART_MAX_TOPK;
  if (total <= 64 * TOPK_MERGE_REGS) {
    uint64_t mine[TOPK_MERGE_REGS];
#pragma unroll
    for (int e = 0; e < TOPK_MERGE_REGS; ++e) {
      const int j = e * 64 + lane;
      mine[e] = j < total ? fetch(&csrc[(size_t)(j / k) * DART_MAX_TOPK + j % k]) : 0;
    }
    wave_select(mine, k, sel[0], emit);
  } else {                                          // very large vocab x k: re-read from memory
    uint64_t bound = ~(uint64_t)0;
    for (int it = 0; it < k; ++it) {
      uint64_t best = 0;
      for (int j = lane; j < total; j += 64) {
        const uint64_t kk = fetch(&csrc[(size_t)(j / k) * DART_MAX_TOPK + j % k]);
        if (kk < bound && kk > best) best = kk;
      }
      best = wave_max_u64(best);
      if (lane == 0) emit(it, best);
      bound = best;
    }
  }
}

hipError_t launch_topk(const dart_ctx *c, const float *logits, int rows, int vocab, int k, float eps,
                       int32_t *ids, float *scores, hipStream_t st) {
  const int nchunks = (vocab + TOPK_CHUNK - 1) / TOPK_CHUNK;
  hipLaunchKernelGGL(topk_kernel, dim3(nchunks, rows), dim3(TOPK_THREADS), 0, st, logits, vocab, k,
                     nchunks, eps, c->topk_cand, c->topk_ms, c->topk_count, ids, scores);
  return hipGetLastError();
}

}  // namespace dart
