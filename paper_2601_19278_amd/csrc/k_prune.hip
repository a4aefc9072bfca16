// Continuity-aware tree pruning (paper Alg. 1, constants and Combine of App. D) on the GPU:
// one workgroup per sequence, the candidate frontier (beam), the level's expansions and
// the running best-theta list all resident in LDS; the N-gram model is a device hash table
// (context -> successor row), one lookup per beam entry serving all k candidates (the
// single-traversal retrieval of App. C.2).
//
// Per level L: every (beam entry b, candidate c) pair is scored
//     inc = ((w_logit[L] * s_logit) + (w_ng * s_ng)) * w_level[L],  score = parent + inc
// with one fp32 rounding per operation (no FMA contraction), so results are bit-identical
// to a CPU evaluation of the same formula.  Each expansion becomes one 64-bit ordering key
//     [ order-preserving score bits : 32 | 15 - level : 4 | 0x0FFFFFFF - creation : 28 ]
// (creation = b*k + c).  Larger key = better under both cuts of the algorithm: within one
// level it orders by (score desc, creation asc) -- the beam cut -- and across levels by
// (score desc, level asc, creation asc) -- the global theta cut.  Ranking the level's keys
// gives the next beam (first w) and the level's contenders for the global tree (first theta),
// which are merged into the running best-theta list.  Since the best theta of a union is the
// best theta of (best theta of one part) + (the other part), the running list equals Alg. 1's
// "top-theta of T" after the last level.  Ways of ranking a level: when a call's levels have at
// most 1024 expansions (the presets: w*k = 200; the paper's defaults: 20 * 25 = 500) -- one
// wavefront selects the max(w, theta) expansions that matter by a threshold search and ranks
// only those (see the kernel); otherwise -- ranking by counting over all threads for the levels
// of up to 1024 expansions (the first ones), a bitonic sort beyond.
//
// N-gram lookups.  The context a beam entry presents at level L is the last N-1 tokens of its
// path: (candidate a of level L-2, candidate b of level L-1) for a trigram.  Which paths
// survive depends on the scores, but the set of contexts that CAN occur does not: it is
// 1 + k + (K-2) k^2 candidate pairs, known from the candidate lists alone.  When that set is
// small enough for LDS (k <= 13 at K = 8), the kernel resolves all of them before the first
// level -- every hash probe and every successor-row read of the call in flight at once, two
// memory round trips in total -- and the K levels then run without touching memory.
// Otherwise, when at least the table rows of all possible contexts fit (k <= 45 at K = 8),
// all hash probes still go out before the first level and a level only fetches the successor
// rows of its own beam entries (at most w per level, as in App. C.2); beyond that each level
// also probes for its beam entries' contexts.
// A loaded successor is matched against its level's k candidates through a small bucketed
// table of the candidate ids in LDS (one 16-byte read per successor instead of k compares).
#include "common.h"
#include "dart_internal.h"

namespace dart {

constexpr int PRUNE_THREADS = 1024;    // one workgroup per sequence; many phases are item-parallel
static_assert(DART_MAX_LEVEL_NODES <= 16384, "a level's pair scores share the ng array");
constexpr int PRUNE_NG_CELLS = 16384;  // N-gram scores of all possible (context, candidate) pairs
constexpr int PRUNE_NG_CTX = 1280;     // possible contexts of one call resolved up front
constexpr int PRUNE_SMALL = 1024;      // expansions per level the short-level loop handles (w * k)

// Short-level mode (at most PRUNE_SMALL expansions per level): the buffers of the wavefront that
// ranks a level.  They share their memory with the expansion keys of the general mode.
struct PruneSmall {
  __align__(16) uint32_t sel_sc[PRUNE_SMALL];  // sortable scores of the level's expansions that matter
  int32_t sel_e[PRUNE_SMALL];                  // ... and their (creation index << 16) | (beam entry << 8) | candidate
  uint8_t pos[DART_MAX_K * PRUNE_SMALL];       // output index of the node (level, creation)
};

struct PruneShared {
  union {
    uint64_t keys[DART_MAX_LEVEL_NODES];      // general mode: this level's expansions (emission: the mask)
    PruneSmall sm;
  };
  int32_t cand_id[DART_MAX_K * DART_MAX_TOPK];
  float cand_sc[DART_MAX_K * DART_MAX_TOPK];
  // beam (double buffered)
  float beam_score[2][DART_MAX_BEAM];
  int32_t beam_tok[2][DART_MAX_BEAM];
  int32_t beam_prev[2][DART_MAX_BEAM];
  int32_t beam_cre[2][DART_MAX_BEAM];          // creation index of the entry at its own level
  int32_t beam_row[DART_MAX_BEAM];             // table row of the entry's context, -1 = unseen
  int32_t rank[PRUNE_THREADS];                 // rank of expansion e among the level's keys
  int32_t beam_ci[2][DART_MAX_BEAM];           // candidate index of the entry's token at its level
  int32_t beam_pi[2][DART_MAX_BEAM];           // candidate index of its parent's token
  // up-front mode: s_ng of candidate c for possible context g at ng[g * k + c];
  // level-by-level mode: s_ng of every (beam entry b, candidate c) pair of the level at
  // ng[b * k + c], filled while the beam entries' successor rows stream in
  float ng[PRUNE_NG_CELLS];
  int32_t ctx_row[PRUNE_NG_CTX];               // table row of possible context g, -1 = unseen
  int32_t hit_ctx[PRUNE_NG_CTX];               // the contexts that have a row
  int32_t n_hit;
  // the level's best min(theta, n_new) expansions, sorted by key descending
  uint64_t lvl_key[2][DART_MAX_BUDGET];       // ([0] only, outside the short-level mode)
  int32_t lvl_tok[2][DART_MAX_BUDGET];
  int32_t lvl_par[2][DART_MAX_BUDGET];
  // running best list (double buffered), sorted by key descending
  uint64_t best_key[2][DART_MAX_BUDGET];
  int32_t best_tok[2][DART_MAX_BUDGET];
  int32_t best_par[2][DART_MAX_BUDGET];        // creation index of the parent at level-1
  // candidate ids of every level in a bucketed table (cand_buckets() buckets of four ids per
  // level): which candidate of level L, if any, is token id?  One 16-byte read answers it.
  __align__(16) int32_t ch_id[DART_MAX_K * DART_MAX_TOPK * 4];   // -1 = empty
  uint8_t ch_c[DART_MAX_K * DART_MAX_TOPK * 4];
  int32_t ch_over[DART_MAX_K];                  // a bucket of the level overflowed: search linearly
  // emission
  int32_t out_idx[DART_MAX_BUDGET];
  int32_t out_par[DART_MAX_BUDGET];
  // short-level mode
  __align__(16) uint32_t lvl_sc[2][DART_MAX_BUDGET];   // scores of lvl_key[][], padded with 0 to a multiple of 4
  __align__(16) uint32_t best_sc[2][DART_MAX_BUDGET];  // scores of best_key[][], likewise
  int32_t lvl_cnt[2][DART_MAX_K];              // selected nodes per level, per wavefront
};

static_assert(sizeof(PruneShared) <= 160 * 1024, "one workgroup's state must fit the 160 KiB of LDS");

__device__ __forceinline__ uint64_t pack_context(int ctx_len, int prev, int tok) {
  return ctx_len >= 2 ? ((uint64_t)(uint32_t)prev << 32) | (uint32_t)tok : (uint64_t)(uint32_t)tok;
}

__device__ __forceinline__ uint4 slot_load(const NgramTableDev &tab, uint64_t h) {
  return *reinterpret_cast<const uint4 *>(tab.slots + h);          // one 16-byte access
}

// Linear probing from slot h whose content `raw` has already been fetched: row of the packed
// context, or -1.  A table is at most half full and the probe count is bounded by its size,
// so the loop always ends.
__device__ __forceinline__ int32_t ngram_probe(const NgramSlot *slots, uint64_t mask, uint64_t packed, uint64_t h,
                               uint4 raw) {
  for (uint64_t probes = 0; probes <= mask; ++probes) {
    const uint64_t kk = ((uint64_t)raw.y << 32) | raw.x;
    if (kk == packed) return (int32_t)raw.z;
    if (kk == ~(uint64_t)0) return -1;
    h = (h + 1) & mask;
    raw = *reinterpret_cast<const uint4 *>(slots + h);
  }
  return -1;
}

// Back-off (optional): the context without its oldest token, in the lower-order table.  Only a
// trigram table can carry one, so the shorter context is the newest token alone.
__device__ __forceinline__ int32_t ngram_backoff_find(const NgramTableDev &tab, int tok) {
  if (!tab.bo_slots) return -1;
  const uint64_t packed = (uint64_t)(uint32_t)tok;
  const uint64_t h = mix64(packed) & tab.bo_slot_mask;
  const int32_t row = ngram_probe(tab.bo_slots, tab.bo_slot_mask, packed, h,
                                  *reinterpret_cast<const uint4 *>(tab.bo_slots + h));
  return row < 0 ? -1 : (row | NGRAM_BACKOFF_ROW);
}

// Finish a lookup of context (.., tok) whose first slot `raw` (at index h) has already been
// fetched: its row, else its back-off row (flagged), else -1.
__device__ __forceinline__ int32_t ngram_resolve(const NgramTableDev &tab, uint64_t packed, uint64_t h, uint4 raw, int tok) {
  const int32_t row = ngram_probe(tab.slots, tab.slot_mask, packed, h, raw);
  return row >= 0 ? row : ngram_backoff_find(tab, tok);
}

__device__ __forceinline__ int32_t ngram_find(const NgramTableDev &tab, uint64_t packed, int tok) {
  const uint64_t h = mix64(packed) & tab.slot_mask;
  return ngram_resolve(tab, packed, h, slot_load(tab, h), tok);
}

// Successor ids and scores of a row as a lookup reported it.
__device__ __forceinline__ void ngram_row(const NgramTableDev &tab, int32_t row, const int32_t *&ids,
                                          const float *&logp) {
  const bool bo = (row & NGRAM_BACKOFF_ROW) != 0;
  const size_t at = (size_t)(row & (NGRAM_BACKOFF_ROW - 1)) * tab.S;
  ids = (bo ? tab.bo_succ_ids : tab.succ_ids) + at;
  logp = (bo ? tab.bo_succ_logp : tab.succ_logp) + at;
}

__device__ __forceinline__ int key_level(uint64_t key) { return 15 - (int)((key >> 28) & 0xF); }
__device__ __forceinline__ int key_creation(uint64_t key) {
  return 0x0FFFFFFF - (int)(key & 0x0FFFFFFF);
}

// Buckets per level of the candidate table: a power of two >= k.
__device__ __forceinline__ int cand_buckets(int k) {
  int H = 1;
  while (H < k) H <<= 1;
  return H;
}
__device__ __forceinline__ uint32_t cand_hash(int32_t id, int H) {
  return ((uint32_t)id * 2654435761u >> 16) & (uint32_t)(H - 1);
}

// Enter the K*k candidates (ids distinct within a level).  Ends with a barrier.
__device__ __forceinline__ void build_cand_table(PruneShared &sh, int K, int k, int t) {
  const int H = cand_buckets(k);
  for (int i = t; i < K * H * 4; i += PRUNE_THREADS) sh.ch_id[i] = -1;
  if (t < K) sh.ch_over[t] = 0;
  __syncthreads();
  for (int e = t; e < K * k; e += PRUNE_THREADS) {
    const int L = e / k, c = e - L * k;
    const int32_t id = sh.cand_id[e];
    const int base = (L * H + (int)cand_hash(id, H)) * 4;
    bool placed = false;
    for (int s = 0; s < 4 && !placed; ++s)
      if (atomicCAS(&sh.ch_id[base + s], -1, id) == -1) {
        sh.ch_c[base + s] = (uint8_t)c;
        placed = true;
      }
    if (!placed) sh.ch_over[L] = 1;
  }
  __syncthreads();
}

// Index of token id among the candidates of level L, or -1.
__device__ __forceinline__ int cand_find(const PruneShared &sh, int L, int H, int k, int32_t id) {
  if (id < 0) return -1;                                 // unused successor slot
  const int base = (L * H + (int)cand_hash(id, H)) * 4;
  const int4 b = *reinterpret_cast<const int4 *>(&sh.ch_id[base]);
  const int s = b.x == id ? 0 : (b.y == id ? 1 : (b.z == id ? 2 : (b.w == id ? 3 : -1)));
  if (s >= 0) return sh.ch_c[base + s];
  if (sh.ch_over[L])
    for (int c = 0; c < k; ++c)
      if (sh.cand_id[L * k + c] == id) return c;
  return -1;
}

// N-gram scores of level L for the nb current beam entries: s_ng[b*k + c] = stored score of
// candidate c among the successors of beam entry b's context, else the miss score.  The
// successor rows are read once, coalesced, all loads independent; each loaded successor is
// looked up in the level's candidate table.  Successor ids are distinct within a row and
// candidate ids within a level, so at most one thread writes a cell.
__device__ __forceinline__ void score_rows(PruneShared &sh, const NgramTableDev &tab, int nb, int k,
                                           int L, int t) {
  const int S = tab.S, H = cand_buckets(k);
  for (int e = t; e < nb * k; e += PRUNE_THREADS) sh.ng[e] = tab.logp_miss;
  __syncthreads();
  for (int idx = t; idx < nb * S; idx += PRUNE_THREADS) {
    const int b = idx / S, j = idx - b * S;
    const int row = sh.beam_row[b];
    if (row >= 0) {
      const int32_t *rid;
      const float *rlp;
      ngram_row(tab, row, rid, rlp);
      const int32_t id = rid[j];
      const float lp = rlp[j];
      const int c = cand_find(sh, L, H, k, id);
      if (c >= 0) sh.ng[b * k + c] = lp;
    }
  }
}

// Possible contexts, numbered level by level: level 0 has one (the real tail), level 1 has k
// (root, candidate), levels >= 2 have k*k (k for a bigram model, whose context is one token).
__device__ __forceinline__ int ctx_offset(int L, int k, int ctx_len) {
  if (L == 0) return 0;
  if (ctx_len < 2) return 1 + (L - 1) * k;
  return L == 1 ? 1 : 1 + k + (L - 2) * k * k;
}

// Up-front resolution of every possible context (see the header): fills sh.ng.
// Number of entries of a score list that beat a score: entries of blocks below jt count when
// they are >= mine (they win ties), the others when they are > mine.  s4: the list in LDS, n4
// (1..64) groups of four, padded with 0 (scores are > 0).  The order of the count does not
// matter, so every lane starts at a different group and walks the list cyclically: the lanes
// of a wavefront then read different LDS addresses in every step.
__device__ __forceinline__ int count_above(const uint4 *s4, int n4, uint32_t mine, int jt) {
  const int lane = threadIdx.x & 63;
  const uint32_t inv = (65536u + n4 - 1) / n4;
  int idx = lane - (int)(((uint32_t)lane * inv) >> 16) * n4;      // lane mod n4
  int r = 0;
  // four compares into four mask registers, then four add-with-carry: written out because the
  // compiler routes every compare through VCC and pays wait states after each one
  auto add4 = [&](const uint4 &v, uint32_t thr) {
    uint64_t m0, m1, m2, m3;
    asm("v_cmp_gt_u32_e64 %[m0], %[x], %[t]\n\t"
        "v_cmp_gt_u32_e64 %[m1], %[y], %[t]\n\t"
        "v_cmp_gt_u32_e64 %[m2], %[z], %[t]\n\t"
        "v_cmp_gt_u32_e64 %[m3], %[w], %[t]\n\t"
        "v_addc_co_u32_e64 %[r], %[m0], 0, %[r], %[m0]\n\t"
        "v_addc_co_u32_e64 %[r], %[m1], 0, %[r], %[m1]\n\t"
        "v_addc_co_u32_e64 %[r], %[m2], 0, %[r], %[m2]\n\t"
        "v_addc_co_u32_e64 %[r], %[m3], 0, %[r], %[m3]"
        : [r] "+v"(r), [m0] "=&s"(m0), [m1] "=&s"(m1), [m2] "=&s"(m2), [m3] "=&s"(m3)
        : [x] "v"(v.x), [y] "v"(v.y), [z] "v"(v.z), [w] "v"(v.w), [t] "v"(thr));
  };
  auto next = [&](int i) { return i + 1 == n4 ? 0 : i + 1; };
  int j = 0;
  for (; j + 4 <= n4; j += 4) {              // four groups in flight
    const int i0 = idx, i1 = next(i0), i2 = next(i1), i3 = next(i2);
    const uint4 v0 = s4[i0], v1 = s4[i1], v2 = s4[i2], v3 = s4[i3];
    add4(v0, i0 < jt ? mine - 1 : mine);
    add4(v1, i1 < jt ? mine - 1 : mine);
    add4(v2, i2 < jt ? mine - 1 : mine);
    add4(v3, i3 < jt ? mine - 1 : mine);
    idx = next(i3);
  }
  for (; j < n4; ++j) {
    add4(s4[idx], idx < jt ? mine - 1 : mine);
    idx = next(idx);
  }
  return r;
}

// The two newest tokens (prev, tok) of possible context g (numbering of ctx_offset).
__device__ __forceinline__ void context_tokens(const PruneShared &sh, int g, int k, int ctx_len, int prev0,
                                               int root, int &prev, int &tok) {
  int L, idx;
  if (g == 0) {
    L = 0, idx = 0;
  } else if (ctx_len < 2) {
    L = 1 + (g - 1) / k, idx = (g - 1) % k;
  } else if (g < 1 + k) {
    L = 1, idx = g - 1;
  } else {
    L = 2 + (g - 1 - k) / (k * k), idx = (g - 1 - k) % (k * k);
  }
  if (L == 0) {
    prev = prev0, tok = root;
  } else if (ctx_len < 2 || L == 1) {
    prev = root, tok = sh.cand_id[(L - 1) * k + idx];
  } else {
    prev = sh.cand_id[(L - 2) * k + idx / k], tok = sh.cand_id[(L - 1) * k + idx % k];
  }
}

// Table rows of all NC possible contexts into rows[] (-1 = unseen), when the pair scores of all
// of them do not fit LDS but their rows do: the hash probes of the whole call are in flight
// together (four per thread at a time) instead of one dependent probe per level, and a level
// only fetches its beam entries' successor rows.
__device__ __forceinline__ void resolve_context_rows(const PruneShared &sh, const NgramTableDev &tab, int NC, int k,
                                     int ctx_len, int prev0, int root, int t, int32_t *rows) {
  constexpr int Q = 4;
  for (int g0 = 0; g0 < NC; g0 += Q * PRUNE_THREADS) {
    uint64_t packed[Q], hslot[Q];
    uint4 raw[Q];
    int newest[Q];
#pragma unroll
    for (int q = 0; q < Q; ++q) {
      const int g = g0 + q * PRUNE_THREADS + t;
      if (g < NC) {
        int prev, tok;
        context_tokens(sh, g, k, ctx_len, prev0, root, prev, tok);
        packed[q] = pack_context(ctx_len, prev, tok);
        newest[q] = tok;
        hslot[q] = mix64(packed[q]) & tab.slot_mask;
        raw[q] = slot_load(tab, hslot[q]);
      }
    }
#pragma unroll
    for (int q = 0; q < Q; ++q) {
      const int g = g0 + q * PRUNE_THREADS + t;
      if (g < NC) rows[g] = ngram_resolve(tab, packed[q], hslot[q], raw[q], newest[q]);
    }
  }
}

__device__ __forceinline__ void resolve_all_contexts(PruneShared &sh, const NgramTableDev &tab, int K, int k,
                                     int ctx_len, int prev0, int root, int t) {
  const int NC = ctx_offset(K, k, ctx_len);
  for (int e = t; e < NC * k; e += PRUNE_THREADS) sh.ng[e] = tab.logp_miss;
  if (t == 0) sh.n_hit = 0;
  __syncthreads();
  // 1. hash probes, one or two contexts per thread, first slots of all of them in flight together
  constexpr int Q = (PRUNE_NG_CTX + PRUNE_THREADS - 1) / PRUNE_THREADS;
  uint64_t packed[Q], hslot[Q];
  uint4 raw[Q];
  int newest[Q];
#pragma unroll
  for (int q = 0; q < Q; ++q) {
    const int g = t + q * PRUNE_THREADS;
    if (g < NC) {
      int prev, tok;
      context_tokens(sh, g, k, ctx_len, prev0, root, prev, tok);
      packed[q] = pack_context(ctx_len, prev, tok);
      newest[q] = tok;
      hslot[q] = mix64(packed[q]) & tab.slot_mask;
      raw[q] = slot_load(tab, hslot[q]);
    }
  }
#pragma unroll
  for (int q = 0; q < Q; ++q) {
    const int g = t + q * PRUNE_THREADS;
    if (g < NC) {
      const int row = ngram_resolve(tab, packed[q], hslot[q], raw[q], newest[q]);
      sh.ctx_row[g] = row;
      if (row >= 0) {
        const int L = g == 0 ? 0
                      : (ctx_len < 2 ? 1 + (g - 1) / k : (g < 1 + k ? 1 : 2 + (g - 1 - k) / (k * k)));
        sh.hit_ctx[atomicAdd(&sh.n_hit, 1)] = g | (L << 16);   // order irrelevant: cells are disjoint
      }
    }
  }
  __syncthreads();
  // 2. successor rows of the contexts that exist, each successor compared with the k
  //    candidates of the context's level.  Successor ids are distinct within a row and
  //    candidate ids within a level, so at most one thread writes a cell.
  const int S = tab.S, n_hit = sh.n_hit, H = cand_buckets(k);
  bool over_any = false;
  for (int L = 0; L < K; ++L) over_any |= sh.ch_over[L] != 0;
  if ((S & 3) == 0) {
    const int parts = S >> 2;                  // 16-byte pieces per row
    const int total = n_hit * parts;
    // item / parts by a reciprocal: exact while item * parts < 2^20 (items < 1280 * 16)
    const uint32_t inv = ((1u << 20) + parts - 1) / parts;
    constexpr int U = 8;
    for (int i0 = t; i0 < total; i0 += U * PRUNE_THREADS) {
      // all 2*U loads of a thread are issued before the first use; items past the end are
      // clamped (loaded twice, used once) so that no branch separates the loads
      int4 id4[U];
      float4 lp4[U];
      int hc[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int item = min(i0 + u * PRUNE_THREADS, total - 1);
        const int hi = (int)(((uint32_t)item * inv) >> 20), piece = item - hi * parts;
        hc[u] = sh.hit_ctx[hi];
        const int32_t *rid;
        const float *rlp;
        ngram_row(tab, sh.ctx_row[hc[u] & 0xFFFF], rid, rlp);
        id4[u] = *reinterpret_cast<const int4 *>(rid + 4 * piece);
        lp4[u] = *reinterpret_cast<const float4 *>(rlp + 4 * piece);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (i0 + u * PRUNE_THREADS < total) {
          const int g = hc[u] & 0xFFFF, L = hc[u] >> 16;
          const int idv[4] = {id4[u].x, id4[u].y, id4[u].z, id4[u].w};
          const float lpv[4] = {lp4[u].x, lp4[u].y, lp4[u].z, lp4[u].w};
          // the four bucket reads go out together; branches only on a match (rare)
          int base[4], slot[4];
          int4 bk[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            base[r] = (L * H + (int)cand_hash(idv[r], H)) * 4;
            bk[r] = *reinterpret_cast<const int4 *>(&sh.ch_id[base[r]]);
          }
          bool any = false;
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int id = idv[r];
            slot[r] = id < 0 ? -1
                             : (bk[r].x == id ? 0 : (bk[r].y == id ? 1 : (bk[r].z == id ? 2 : (bk[r].w == id ? 3 : -1))));
            any |= slot[r] >= 0;
          }
          if (any) {
#pragma unroll
            for (int r = 0; r < 4; ++r)
              if (slot[r] >= 0) sh.ng[g * k + sh.ch_c[base[r] + slot[r]]] = lpv[r];
          }
          if (over_any && sh.ch_over[L]) {              // a bucket of this level overflowed
#pragma unroll
            for (int r = 0; r < 4; ++r)
              if (slot[r] < 0 && idv[r] >= 0)
                for (int c = 0; c < k; ++c)
                  if (sh.cand_id[L * k + c] == idv[r]) sh.ng[g * k + c] = lpv[r];
          }
        }
      }
    }
  } else {
    for (int item = t; item < n_hit * S; item += PRUNE_THREADS) {
      const int hcx = sh.hit_ctx[item / S];
      const int g = hcx & 0xFFFF, L = hcx >> 16;
      const int32_t *rid;
      const float *rlp;
      ngram_row(tab, sh.ctx_row[g], rid, rlp);
      const int32_t id = rid[item % S];
      const float lp = rlp[item % S];
      const int c = cand_find(sh, L, H, k, id);
      if (c >= 0) sh.ng[g * k + c] = lp;
    }
  }
}

// The level loop of the short-level mode (see the kernel).  NS: scores per lane of the ranking
// wavefront (4 up to 256 expansions per level, 8 up to 512, 16 up to 1024).  PRE: every N-gram score is in LDS
// already (up-front mode); otherwise the scores of a level's pairs are fetched between levels.  nb, n_best, cur, bcur: beam size,
// best-list length and the live halves of the double buffers, carried on to the emission.
template <int NS, bool PRE>
__device__ __forceinline__ void short_levels(PruneShared &sh, const NgramTableDev &tab,
                                             const PruneLevelWeights &lw, int K, int k, int beam_w,
                                             int theta, int ctx_len, float w_ng, bool pre_rows,
                                             const int32_t *rows_all, int t, int &nb, int &n_best,
                                             int &cur, int &bcur) {
  const int lane = t & 63, wav = t >> 6;
  int n_lvl_prev = 0;
  // Both lists are sorted and the level list's entries all have a higher level than the best
  // list's, so between the lists the score decides and a tie goes to the best list's entry.
  // Done by threads 64 .. 64 + n_best + n_lvl_prev (at most 2 * 127 of them).
  auto merge_prev = [&](int lb) {
    const int bnx = bcur ^ 1;
    const int n_out = min(theta, n_best + n_lvl_prev);
    const int tt = t - 64;
    if (tt >= 0 && tt < n_best + n_lvl_prev) {
      uint64_t key;
      uint32_t sc;
      int tok, par, rank;
      if (tt < n_best) {
        key = sh.best_key[bcur][tt];
        sc = sh.best_sc[bcur][tt];
        tok = sh.best_tok[bcur][tt];
        par = sh.best_par[bcur][tt];
        rank = tt + count_above(reinterpret_cast<const uint4 *>(sh.lvl_sc[lb]),
                                (n_lvl_prev + 3) >> 2, sc, 0);
      } else {
        const int j0 = tt - n_best;
        key = sh.lvl_key[lb][j0];
        sc = sh.lvl_sc[lb][j0];
        tok = sh.lvl_tok[lb][j0];
        par = sh.lvl_par[lb][j0];
        const int b4 = (n_best + 3) >> 2;
        rank = j0 + (n_best ? count_above(reinterpret_cast<const uint4 *>(sh.best_sc[bcur]), b4, sc, b4) : 0);
        if (sc == 0) rank = theta;                       // an entry the level did not keep
      }
      if (rank < theta) {
        sh.best_key[bnx][rank] = key;
        sh.best_sc[bnx][rank] = sc;
        sh.best_tok[bnx][rank] = tok;
        sh.best_par[bnx][rank] = par;
      }
    } else if (t >= 512 && t - 512 + n_out < ((n_out + 3) & ~3)) {
      sh.best_sc[bnx][t - 512 + n_out] = 0;              // padding of the merged list
    }
    n_best = n_out;
    bcur = bnx;
  };
  for (int L = 0; L < K; ++L) {
    const int n_new = nb * k;
    const int nb_next = min(beam_w, n_new);
    const int n_lvl = min(theta, n_new);
    const int nxt = cur ^ 1, lb = L & 1;
    const bool last = L + 1 == K;
    if (wav == 0) {
      const float wl = lw.w_logit[L], wv = lw.w_level[L];
      // scores of expansions lane, lane + 64, ... (0 = none).  Indices are clamped instead of
      // branched on, so that the dependent LDS chains overlap; e / k by a reciprocal (exact for
      // e < 1024, k <= 64: checked exhaustively).
      uint32_t sc[NS];
      int bc[NS];                             // (beam entry << 8) | candidate
      const uint32_t inv_k = (65536u + k - 1) / k;
#pragma unroll
      for (int i = 0; i < NS; ++i) {
        const int e = min(lane + 64 * i, n_new - 1);
        const int bb = (int)(((uint32_t)e * inv_k) >> 16), c = e - bb * k;
        const int p_ci = sh.beam_ci[cur][bb];
        const int gctx = ctx_offset(L, k, ctx_len) +
                         (L < 2 || ctx_len < 2 ? p_ci : sh.beam_pi[cur][bb] * k + p_ci);
        const float a = __fmul_rn(wl, sh.cand_sc[L * k + c]);
        const float g = __fmul_rn(w_ng, sh.ng[PRE ? gctx * k + c : e]);
        const float inc = __fmul_rn(__fadd_rn(a, g), wv);
        const uint32_t v = f32_sortable(__fadd_rn(sh.beam_score[cur][bb], inc));
        sc[i] = lane + 64 * i < n_new ? v : 0;
        bc[i] = (bb << 8) | c;
      }
      // Once the best list is full, its last score is a floor: an expansion at or below it
      // can never enter the tree (a tie goes to the lower level), so the level list needs
      // only the expansions above the floor.  The list as merged two levels ago is the one
      // this wavefront may read; its floor is lower than the current one, which is safe.
      int n_keep = n_lvl;
      if (theta > 0 && n_best == theta) {
        const uint32_t floor_sc = sh.best_sc[bcur][theta - 1];
        int above_floor = 0;
#pragma unroll
        for (int i = 0; i < NS; ++i) above_floor += (int)__popcll(__ballot(sc[i] > floor_sc));
        n_keep = min(n_lvl, above_floor);
      }
      const int need = max(nb_next, n_keep);   // expansions of this level that matter (<= n_new)
      // A threshold T with at least `need` scores >= T, found bit by bit from the top (every
      // accepted bit keeps that property).  The search stops as soon as few more than `need`
      // scores are left above T: any such T selects a superset of the expansions that matter.
      // The bits that all scores of the level share (sign, exponent and often the first
      // mantissa bits) are taken over at once: T starts as that common prefix, which is <= every
      // score, and the search begins at the highest bit in which two scores differ.
      uint32_t hi = 0, lo = ~0u;
#pragma unroll
      for (int i = 0; i < NS; ++i) {
        hi = max(hi, sc[i]);
        lo = min(lo, sc[i] ? sc[i] : ~0u);
      }
      const uint32_t top = wave_max_u32(hi);
      const uint32_t bot = ~wave_max_u32(~lo);
      const int first = 31 - __clz((int)(top ^ bot));           // -1: all scores are equal
      uint32_t T = first < 0 ? top : top & ~((2u << first) - 1u);
      int above = n_new;
      const int enough = need <= 64 ? 64 : need + 8;   // up to 64 are ranked in one pass
      for (int bit = first; bit >= 0 && above > enough; --bit) {
        const uint32_t trial = T | (1u << bit);
        int cnt = 0;
#pragma unroll
        for (int i = 0; i < NS; ++i) cnt += (int)__popcll(__ballot(sc[i] >= trial));
        if (cnt >= need) {
          T = trial;
          above = cnt;
        }
      }
      // the expansions with score >= T (real scores are > 0, T >= the smallest of them), in
      // creation order
      int m = 0;
#pragma unroll
      for (int i = 0; i < NS; ++i) {
        const bool in = sc[i] >= T && sc[i] != 0;
        const uint64_t mask = __ballot(in);
        if (in) {
          const int at = m + __popcll(mask & (((uint64_t)1 << lane) - 1));
          sh.sm.sel_sc[at] = sc[i];
          sh.sm.sel_e[at] = ((lane + 64 * i) << 16) | bc[i];
        }
        m += __popcll(mask);
      }
      if (lane < ((m + 3) & ~3) - m) sh.sm.sel_sc[m + lane] = 0;      // pad the last group of four
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      // rank among the selected = rank among all: scores above mine + equal scores created
      // before me (= earlier in the list)
      const uint4 *s4 = reinterpret_cast<const uint4 *>(sh.sm.sel_sc);
      for (int p0 = lane; p0 < m; p0 += 64) {
        const uint32_t mine = sh.sm.sel_sc[p0];
        const int ebc = sh.sm.sel_e[p0];
        const int e = ebc >> 16, bb = (ebc >> 8) & 0xFF, c = ebc & 0xFF;
        const int jt = p0 >> 2;
        int r = count_above(s4, (m + 3) >> 2, mine, jt);
        {
          const uint4 v = s4[jt];                        // my own group: ties before me
          const int i = p0 & 3;
          r += (i > 0 && v.x == mine) + (i > 1 && v.y == mine) + (i > 2 && v.z == mine);
        }
        if (r < need) {
          const int tok = sh.cand_id[L * k + c];
          if (r < nb_next) {
            sh.beam_score[nxt][r] = f32_unsortable(mine);
            sh.beam_tok[nxt][r] = tok;
            sh.beam_prev[nxt][r] = sh.beam_tok[cur][bb];
            sh.beam_cre[nxt][r] = e;
            sh.beam_ci[nxt][r] = c;
            sh.beam_pi[nxt][r] = sh.beam_ci[cur][bb];
            if (!PRE && !last) {                         // table row of the context it will present
              const int gnext = ctx_offset(L + 1, k, ctx_len) +
                                (L + 1 < 2 || ctx_len < 2 ? c : sh.beam_ci[cur][bb] * k + c);
              sh.beam_row[r] = pre_rows ? rows_all[gnext]
                                        : ngram_find(tab, pack_context(ctx_len, sh.beam_tok[cur][bb], tok), tok);
            }
          }
          if (r < n_keep) {
            sh.lvl_key[lb][r] = ((uint64_t)mine << 32) | ((uint64_t)(15 - L) << 28) |
                                (uint64_t)(0x0FFFFFFF - e);
            sh.lvl_sc[lb][r] = mine;
            sh.lvl_tok[lb][r] = tok;
            sh.lvl_par[lb][r] = sh.beam_cre[cur][bb];
          }
        }
      }
      // the entries not kept and the padding of the last group of four: score 0, which the
      // merge ranks below every real entry
      for (int j = n_keep + lane; j < ((n_lvl + 3) & ~3); j += 64) sh.lvl_sc[lb][j] = 0;
      // the next level's scores read what this level placed
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    if (L > 0) merge_prev(lb ^ 1);
    __syncthreads();
    if (!PRE && !last) {                  // N-gram scores of the next level's (beam entry, candidate) pairs
      score_rows(sh, tab, nb_next, k, L + 1, t);
      __syncthreads();
    }
    n_lvl_prev = n_lvl;
    cur = nxt;
    nb = nb_next;
  }
  merge_prev((K - 1) & 1);
  __syncthreads();
}

__global__ __launch_bounds__(PRUNE_THREADS) void prune_kernel(
    const int32_t *__restrict__ ids, const float *__restrict__ scores, int K,
    const int32_t *__restrict__ ctx_tail, NgramTableDev tab, int k, int beam_w, int budget,
    float w_ng, PruneLevelWeights lw, int32_t *__restrict__ tokens_out,
    int32_t *__restrict__ parents_out, uint8_t *__restrict__ mask_out,
    int32_t *__restrict__ n_nodes_out) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  PruneShared &sh = *reinterpret_cast<PruneShared *>(smem_raw);
  const int seq = blockIdx.x, t = threadIdx.x;
  const int theta = budget - 1;
  const int ctx_len = tab.n_gram - 1;
  ids += (size_t)seq * K * k;
  scores += (size_t)seq * K * k;
  ctx_tail += (size_t)seq * ctx_len;
  tokens_out += (size_t)seq * budget;
  parents_out += (size_t)seq * budget;
  mask_out += (size_t)seq * budget * budget;

  for (int e = t; e < K * k; e += PRUNE_THREADS) {
    sh.cand_id[e] = ids[e];
    sh.cand_sc[e] = scores[e];
  }
  const int root = ctx_tail[ctx_len - 1];
  const int prev0 = ctx_len >= 2 ? ctx_tail[ctx_len - 2] : 0;
  // all possible contexts up front when they fit (uniform for the workgroup)
  const int NC = ctx_offset(K, k, ctx_len);
  const bool pre = NC <= PRUNE_NG_CTX && NC * k <= PRUNE_NG_CELLS;
  // otherwise at least the rows of all possible contexts, when they fit behind the pair scores
  // of one level (at most DART_MAX_LEVEL_NODES cells of ng are used level by level)
  const bool pre_rows = !pre && NC <= PRUNE_NG_CELLS - DART_MAX_LEVEL_NODES;
  int32_t *const rows_all = reinterpret_cast<int32_t *>(sh.ng + DART_MAX_LEVEL_NODES);
  if (t == 0) {
    sh.beam_score[0][0] = 0.f;
    sh.beam_tok[0][0] = root;
    sh.beam_prev[0][0] = prev0;
    sh.beam_cre[0][0] = -1;                    // the root
    sh.beam_ci[0][0] = 0;
    sh.beam_pi[0][0] = 0;
    if (!pre && !pre_rows) sh.beam_row[0] = ngram_find(tab, pack_context(ctx_len, prev0, root), root);
  }
  int nb = 1, n_best = 0, cur = 0, bcur = 0;
  __syncthreads();
  build_cand_table(sh, K, k, t);
  if (pre) {
    resolve_all_contexts(sh, tab, K, k, ctx_len, prev0, root, t);
  } else {
    if (pre_rows) {
      resolve_context_rows(sh, tab, NC, k, ctx_len, prev0, root, t, rows_all);
      __syncthreads();
      if (t == 0) sh.beam_row[0] = rows_all[0];
      __syncthreads();
    }
    score_rows(sh, tab, 1, k, 0, t);
  }
  __syncthreads();

  // Short-level mode: every level has at most PRUNE_SMALL expansions.  Ranking all w*k expansions
  // of a level by counting costs (w*k)^2 compares (and as many LDS reads), but only the best
  // max(w, theta) of them are ever used.  So one wavefront holds the level's scores in registers
  // (4, 8 or 16 per lane), finds a score T at or just below that of
  // the last expansion that matters by a bitwise search with ballots, compacts the expansions with
  // score >= T into LDS in creation order and ranks only those among themselves (32-bit
  // sortable scores, read four at a time; among equal scores the earlier creation wins, as in
  // the 64-bit key).  Two other wavefronts merge the previous level's list into the best list
  // meanwhile (the level lists are double buffered).  With every N-gram score already in LDS
  // (up-front mode) that wavefront runs the whole beam recursion and a level costs one barrier;
  // otherwise it also notes the table rows of the next beam, and all threads fetch those rows'
  // successors between two levels (score_rows).
  const bool small = beam_w * k <= PRUNE_SMALL;
  if (small) {
#define DART_SHORT_LEVELS(NS_, PRE_)                                                                  \
  short_levels<NS_, PRE_>(sh, tab, lw, K, k, beam_w, theta, ctx_len, w_ng, pre_rows, rows_all, t, nb, \
                          n_best, cur, bcur)
    if (beam_w * k <= 256) {
      if (pre) DART_SHORT_LEVELS(4, true);
      else DART_SHORT_LEVELS(4, false);
    } else if (beam_w * k <= 512) {
      if (pre) DART_SHORT_LEVELS(8, true);
      else DART_SHORT_LEVELS(8, false);
    } else {
      if (pre) DART_SHORT_LEVELS(16, true);
      else DART_SHORT_LEVELS(16, false);
    }
#undef DART_SHORT_LEVELS
  }

  for (int L = 0; !small && L < K; ++L) {
    const int n_new = nb * k;
    const int nb_next = min(beam_w, n_new);
    const int n_lvl = min(theta, n_new);
    const int nxt = cur ^ 1;
    const bool last = L + 1 == K;
    const float wl = lw.w_logit[L], wv = lw.w_level[L];

    // score of expansion e = b*k + c of this level as its ordering key
    auto expansion_key = [&](int e, int &tok_out, int &b_out) -> uint64_t {
      const int b = e / k, c = e - b * k;
      const int tok = sh.cand_id[L * k + c];
      // up-front mode: the entry's context is (its parent's candidate, its own candidate)
      const int gctx = ctx_offset(L, k, ctx_len) +
                       (L < 2 || ctx_len < 2 ? sh.beam_ci[cur][b]
                                             : sh.beam_pi[cur][b] * k + sh.beam_ci[cur][b]);
      const float s_ng = pre ? sh.ng[gctx * k + c] : sh.ng[e];
      const float a = __fmul_rn(wl, sh.cand_sc[L * k + c]);
      const float g = __fmul_rn(w_ng, s_ng);
      const float inc = __fmul_rn(__fadd_rn(a, g), wv);
      const float sc = __fadd_rn(sh.beam_score[cur][b], inc);
      tok_out = tok;
      b_out = b;
      return ((uint64_t)f32_sortable(sc) << 32) | ((uint64_t)(15 - L) << 28) |
             (uint64_t)(0x0FFFFFFF - e);
    };

    // possible-context number that candidate c of this level, expanded from beam entry b, presents
    // at the next level: (its parent's candidate, its own candidate)
    auto next_context = [&](int c, int b) {
      return ctx_offset(L + 1, k, ctx_len) + (L + 1 < 2 || ctx_len < 2 ? c : sh.beam_ci[cur][b] * k + c);
    };

    if (n_new <= PRUNE_THREADS) {
      // Register-resident path: thread e (< n_new) owns expansion e.  Keys are ranked by
      // counting the keys that beat them (keys are unique); with few expansions the count of
      // one key is split over PARTS threads (thread e + i*span counts slice i of the keys),
      // which shortens the serial loop the level's latency is made of.  In level-by-level
      // mode the owner knows the context its expansion would present at the next level and
      // fetches that context's hash slot before ranking, so the probe overlaps with it.
      const int span = n_new <= PRUNE_THREADS / 4 ? PRUNE_THREADS / 4
                       : (n_new <= PRUNE_THREADS / 2 ? PRUNE_THREADS / 2 : PRUNE_THREADS);
      const int parts = PRUNE_THREADS / span;
      const int e = t % span, part = t / span;
      const bool owner = part == 0 && e < n_new;
      uint64_t key = 0, packed = 0, hslot = 0;
      uint4 raw = make_uint4(0, 0, 0, 0);
      int tok = 0, bb = 0;
      if (owner) {
        key = expansion_key(e, tok, bb);
        sh.keys[e] = key;
        sh.rank[e] = 0;
        if (!last && !pre && !pre_rows) {
          packed = pack_context(ctx_len, sh.beam_tok[cur][bb], tok);
          hslot = mix64(packed) & tab.slot_mask;
          raw = slot_load(tab, hslot);
        }
      }
      __syncthreads();
      if (e < n_new) {
        const uint64_t mine = sh.keys[e];
        const int per = (n_new + parts - 1) / parts;
        const int j0 = part * per, j1 = min(n_new, j0 + per);
        int cnt = 0;
        // (unrolled: eight independent LDS reads in flight instead of one latency per key)
#pragma unroll 8
        for (int j = j0; j < j1; ++j) cnt += sh.keys[j] > mine;
        if (cnt) atomicAdd(&sh.rank[e], cnt);
      }
      __syncthreads();
      int r = PRUNE_THREADS;
      if (owner) {
        r = sh.rank[e];
        if (r < nb_next) {
          sh.beam_score[nxt][r] = f32_unsortable((uint32_t)(key >> 32));
          sh.beam_tok[nxt][r] = tok;
          sh.beam_prev[nxt][r] = sh.beam_tok[cur][bb];
          sh.beam_cre[nxt][r] = e;
          sh.beam_ci[nxt][r] = e - bb * k;
          sh.beam_pi[nxt][r] = sh.beam_ci[cur][bb];
        }
        if (r < n_lvl) {
          sh.lvl_key[0][r] = key;
          sh.lvl_tok[0][r] = tok;
          sh.lvl_par[0][r] = sh.beam_cre[cur][bb];
        }
      }
      // beam_row of this level was last read before the barriers above: safe to overwrite
      if (owner && !last && !pre && r < nb_next)
        sh.beam_row[r] = pre_rows ? rows_all[next_context(e - bb * k, bb)]
                                  : ngram_resolve(tab, packed, hslot, raw, tok);
    } else {
      // General path (up to 4096 expansions): bitonic sort of the keys in LDS.
      int P = 2, logP = 1;
      while (P < n_new) {
        P <<= 1;
        ++logP;
      }
      for (int e = t; e < P; e += PRUNE_THREADS) {
        int tok, b;
        sh.keys[e] = e < n_new ? expansion_key(e, tok, b) : 0;
      }
      __syncthreads();
      for (int ls = 1; ls <= logP; ++ls) {               // size = 1 << ls
        for (int lst = ls - 1; lst >= 0; --lst) {        // stride = 1 << lst
          for (int e = t; e < (P >> 1); e += PRUNE_THREADS) {
            const int lo = ((e >> lst) << (lst + 1)) | (e & ((1 << lst) - 1));
            const int hi = lo + (1 << lst);
            const bool desc = ((lo >> ls) & 1) == 0;
            const uint64_t a = sh.keys[lo], b = sh.keys[hi];
            if (desc ? (a < b) : (a > b)) {
              sh.keys[lo] = b;
              sh.keys[hi] = a;
            }
          }
          __syncthreads();
        }
      }
      int row = -1;
      if (t < max(nb_next, n_lvl)) {
        const uint64_t kk = sh.keys[t];
        const int e = key_creation(kk);
        const int b = e / k, c = e - b * k;
        const int tk = sh.cand_id[L * k + c];
        if (t < nb_next) {
          sh.beam_score[nxt][t] = f32_unsortable((uint32_t)(kk >> 32));
          sh.beam_tok[nxt][t] = tk;
          sh.beam_prev[nxt][t] = sh.beam_tok[cur][b];
          sh.beam_cre[nxt][t] = e;
          sh.beam_ci[nxt][t] = c;
          sh.beam_pi[nxt][t] = sh.beam_ci[cur][b];
          if (!last && !pre)
            row = pre_rows ? rows_all[next_context(c, b)]
                           : ngram_find(tab, pack_context(ctx_len, sh.beam_tok[cur][b], tk), tk);
        }
        if (t < n_lvl) {
          sh.lvl_key[0][t] = kk;
          sh.lvl_tok[0][t] = tk;
          sh.lvl_par[0][t] = sh.beam_cre[cur][b];
        }
      }
      __syncthreads();
      if (t < nb_next) sh.beam_row[t] = row;
    }
    __syncthreads();

    // merge the level's best into the running best list (both sorted, keys unique), and
    // stage the next level's successor rows
    const int bnx = bcur ^ 1;
    if (t < n_best + n_lvl) {
      uint64_t key;
      int tok, par, rank;
      if (t < n_best) {
        key = sh.best_key[bcur][t];
        tok = sh.best_tok[bcur][t];
        par = sh.best_par[bcur][t];
        rank = t;
#pragma unroll 8
        for (int j = 0; j < n_lvl; ++j) rank += (sh.lvl_key[0][j] > key);
      } else {
        const int j0 = t - n_best;
        key = sh.lvl_key[0][j0];
        tok = sh.lvl_tok[0][j0];
        par = sh.lvl_par[0][j0];
        rank = j0;
#pragma unroll 8
        for (int j = 0; j < n_best; ++j) rank += (sh.best_key[bcur][j] > key);
      }
      if (rank < theta) {
        sh.best_key[bnx][rank] = key;
        sh.best_tok[bnx][rank] = tok;
        sh.best_par[bnx][rank] = par;
      }
    }
    if (!last && !pre) score_rows(sh, tab, nb_next, k, L + 1, t);
    n_best = min(theta, n_best + n_lvl);
    bcur = bnx;
    cur = nxt;
    nb = nb_next;
    __syncthreads();
  }

  // emission: root, then level-major; inside a level the best list's order already is
  // (score desc, creation asc)
  const int n_nodes = 1 + n_best;
  if (small) {
    // Output index = 1 + selected nodes of lower levels + my place among those of my level
    // (ballots: at most 127 selected nodes, two wavefronts); the parent's index is then looked
    // up by (level, creation), 0xFF = not selected.
    const int wav = t >> 6, lane = t & 63;
    uint64_t key = 0;
    int lev = -1, within = 0;
    if (t < n_best) {
      key = sh.best_key[bcur][t];
      lev = key_level(key);
    }
    if (t < 128) {
      for (int l = 0; l < K; ++l) {
        const uint64_t m = __ballot(lev == l);
        if (lev == l) within = __popcll(m & (((uint64_t)1 << lane) - 1));
        if (lane == 0) sh.lvl_cnt[wav][l] = __popcll(m);
      }
    }
    for (int i = t; i < K * PRUNE_SMALL / 16; i += PRUNE_THREADS)
      reinterpret_cast<uint4 *>(sh.sm.pos)[i] = make_uint4(~0u, ~0u, ~0u, ~0u);
    __syncthreads();
    if (t < n_best) {
      int idx = 1 + within + (wav == 1 ? sh.lvl_cnt[0][lev] : 0);
      for (int l = 0; l < lev; ++l) idx += sh.lvl_cnt[0][l] + sh.lvl_cnt[1][l];
      sh.out_idx[t] = idx;
      sh.sm.pos[lev * PRUNE_SMALL + key_creation(key)] = (uint8_t)idx;
    }
    __syncthreads();
    if (t < n_best) {
      int parent = 0;
      if (lev > 0) {
        const int v = sh.sm.pos[(lev - 1) * PRUNE_SMALL + sh.best_par[bcur][t]];
        parent = v == 0xFF ? -2 : v;                   // -2 only if the set were not ancestor-closed
      }
      const int idx = sh.out_idx[t];
      sh.out_par[idx] = parent;
      tokens_out[idx] = sh.best_tok[bcur][t];
      parents_out[idx] = parent;
    }
  } else {
    if (t < n_best) {
      const int lev = key_level(sh.best_key[bcur][t]);
      int idx = 1;
#pragma unroll 8
      for (int j = 0; j < n_best; ++j) {
        const int lj = key_level(sh.best_key[bcur][j]);
        idx += (lj < lev) || (lj == lev && j < t);
      }
      sh.out_idx[t] = idx;
    }
    __syncthreads();
    if (t < n_best) {
      const uint64_t key = sh.best_key[bcur][t];
      const int lev = key_level(key);
      int parent = 0;
      if (lev > 0) {
        parent = -2;                                   // stays -2 only if the set were not ancestor-closed
        const int want = sh.best_par[bcur][t];
#pragma unroll 8
        for (int j = 0; j < n_best; ++j) {
          const uint64_t kj = sh.best_key[bcur][j];
          if (key_level(kj) == lev - 1 && key_creation(kj) == want) parent = sh.out_idx[j];
        }
      }
      const int idx = sh.out_idx[t];
      sh.out_par[idx] = parent;
      tokens_out[idx] = sh.best_tok[bcur][t];
      parents_out[idx] = parent;
    }
  }
  if (t == 0) {
    sh.out_par[0] = -1;
    tokens_out[0] = root;
    parents_out[0] = -1;
    n_nodes_out[seq] = n_nodes;
  }
  for (int i = n_nodes + t; i < budget; i += PRUNE_THREADS) {
    tokens_out[i] = -1;
    parents_out[i] = -1;
  }
  // ancestor mask: built in LDS (the expansion keys are no longer needed), written out once
  uint8_t *mk = reinterpret_cast<uint8_t *>(sh.keys);
  const int cells = budget * budget;
  __syncthreads();                     // short-level mode: pos[] lives in the same memory and was just read
  for (int i = t; i < (cells + 3) / 4; i += PRUNE_THREADS) reinterpret_cast<uint32_t *>(mk)[i] = 0;
  __syncthreads();
  if (t < n_nodes) {
    int j = t;
    for (int hops = 0; j >= 0 && hops <= DART_MAX_K; ++hops) {   // depth <= K: bounded walk
      mk[t * budget + j] = 1;
      j = sh.out_par[j];
    }
  }
  __syncthreads();
  if ((cells & 3) == 0 && (reinterpret_cast<uintptr_t>(mask_out) & 3) == 0) {
    for (int i = t; i < cells / 4; i += PRUNE_THREADS)
      reinterpret_cast<uint32_t *>(mask_out)[i] = reinterpret_cast<const uint32_t *>(mk)[i];
  } else {
    for (int i = t; i < cells; i += PRUNE_THREADS) mask_out[i] = mk[i];
  }
}

hipError_t launch_prune(int batch, const int32_t *ids, const float *scores, int K,
                        const int32_t *ctx_tail, const NgramTableDev &tab,
                        const dart_prune_params &p, const PruneLevelWeights &lw, int32_t *tokens,
                        int32_t *parents, uint8_t *mask, int32_t *n_nodes, hipStream_t st) {
  hipError_t e = raise_dynamic_lds_once((const void *)prune_kernel, (int)sizeof(PruneShared));
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(prune_kernel, dim3(batch), dim3(PRUNE_THREADS), sizeof(PruneShared), st, ids,
                     scores, K, ctx_tail, tab, p.k, p.beam_w, p.budget, p.w_ng, lw, tokens, parents,
                     mask, n_nodes);
  return hipGetLastError();
}

}  // namespace dart
