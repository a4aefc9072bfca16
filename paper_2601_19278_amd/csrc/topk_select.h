// Wavefront-level selection of the k largest keys, shared by the top-k kernels and by the LM-head
// kernel that selects its workgroup's candidates itself (Alg. 1 "Top-k_i tokens from l_i").
// Ordering key: (logit descending, token id ascending) as one 64-bit integer
// (order-preserving float map << 32 | ~id), unique per entry.
#pragma once
#include "common.h"

namespace dart {

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

// The same selection for a wavefront's slice of a logit row: the lane's e-th value v[e] is the
// order-preserving word of the logit with vocabulary index index_of(e), valid for e < ne.  The
// 64-bit keys are built only for the few entries that reach the candidate buffer.
template <int N, typename IndexOf, typename Emit>
__device__ __forceinline__ void wave_select_indexed(const uint32_t (&v)[N], int ne, IndexOf index_of, int k,
                                                    uint64_t *buf, Emit emit) {
  const int lane = threadIdx.x & 63;
  uint32_t hm = 0;
#pragma unroll
  for (int e = 0; e < N; ++e) hm = max(hm, e < ne ? v[e] : 0u);
  uint32_t T = 0;
  for (int bit = 31; bit >= 16; --bit) {
    const uint32_t trial = T | (1u << bit);
    if (__popcll(__ballot(hm >= trial)) >= k) T = trial;
  }
  int c = 0;
#pragma unroll
  for (int e = 0; e < N; ++e) c += e < ne && v[e] >= T;
  const int incl = wave_scan_add_dpp(c);
  const int m = __builtin_amdgcn_readlane(incl, 63);
  auto key_of = [&](int e) { return ((uint64_t)v[e] << 32) | (uint32_t)(~(uint32_t)index_of(e)); };
  if (m > TOPK_CAP) {                    // heavy ties: sequential extraction over full keys
    uint64_t key[N];
#pragma unroll
    for (int e = 0; e < N; ++e) key[e] = e < ne ? key_of(e) : 0;
    wave_extract(key, k, [&](int it, uint64_t best) {
      if (lane == 0) emit(it, best);
    });
    return;
  }
  int at = incl - c;
#pragma unroll
  for (int e = 0; e < N; ++e)
    if (e < ne && v[e] >= T) buf[at++] = key_of(e);
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

// ... for entries at indices idx0 + 64 * e (idx0 already includes the lane).
template <int N, typename Emit>
__device__ __forceinline__ void wave_select_row(const uint32_t (&v)[N], int ne, int idx0, int k,
                                                uint64_t *buf, Emit emit) {
  wave_select_indexed(v, ne, [&](int e) { return idx0 + 64 * e; }, k, buf, emit);
}

}  // namespace dart
