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
// (by counting for up to 512 expansions, by a bitonic sort beyond) gives the next beam
// (first w) and the level's contenders for the global tree (first theta), which are merged
// into the running best-theta list.  Since the best
// theta of a union is the best theta of (best theta of one part) + (the other part), the
// running list equals Alg. 1's "top-theta of T" after the last level.
#include "common.h"
#include "dart_internal.h"

namespace dart {

constexpr int PRUNE_THREADS = 256;
constexpr int PRUNE_FAST = 2;          // expansions per thread on the register-resident path

struct PruneShared {
  uint64_t keys[DART_MAX_LEVEL_NODES];        // this level's expansions
  int32_t cand_id[DART_MAX_K * DART_MAX_TOPK];
  float cand_sc[DART_MAX_K * DART_MAX_TOPK];
  // beam (double buffered)
  float beam_score[2][DART_MAX_BEAM];
  int32_t beam_tok[2][DART_MAX_BEAM];
  int32_t beam_prev[2][DART_MAX_BEAM];
  int32_t beam_cre[2][DART_MAX_BEAM];          // creation index of the entry at its own level
  int32_t beam_row[DART_MAX_BEAM];             // table row of the entry's context, -1 = unseen
  // N-gram score of every (beam entry, candidate) pair of the level, filled while the beam
  // entries' successor rows stream in
  float s_ng[DART_MAX_LEVEL_NODES];
  // the level's best min(theta, n_new) expansions, sorted by key descending
  uint64_t lvl_key[DART_MAX_BUDGET];
  int32_t lvl_tok[DART_MAX_BUDGET];
  int32_t lvl_par[DART_MAX_BUDGET];
  // running best list (double buffered), sorted by key descending
  uint64_t best_key[2][DART_MAX_BUDGET];
  int32_t best_tok[2][DART_MAX_BUDGET];
  int32_t best_par[2][DART_MAX_BUDGET];        // creation index of the parent at level-1
  // emission
  int32_t out_idx[DART_MAX_BUDGET];
  int32_t out_par[DART_MAX_BUDGET];
};

__device__ __forceinline__ uint64_t pack_context(int ctx_len, int prev, int tok) {
  return ctx_len >= 2 ? ((uint64_t)(uint32_t)prev << 32) | (uint32_t)tok : (uint64_t)(uint32_t)tok;
}

__device__ __forceinline__ uint4 slot_load(const NgramTableDev &tab, uint64_t h) {
  return *reinterpret_cast<const uint4 *>(tab.slots + h);          // one 16-byte access
}

// Finish a lookup whose first slot `raw` (at index h) has already been fetched: row of the
// packed context, or -1.  Linear probing; the table is at most half full and the probe
// count is bounded by the table size, so the loop always ends.
__device__ int32_t ngram_resolve(const NgramTableDev &tab, uint64_t packed, uint64_t h, uint4 raw) {
  for (uint64_t probes = 0; probes <= tab.slot_mask; ++probes) {
    const uint64_t kk = ((uint64_t)raw.y << 32) | raw.x;
    if (kk == packed) return (int32_t)raw.z;
    if (kk == ~(uint64_t)0) return -1;
    h = (h + 1) & tab.slot_mask;
    raw = slot_load(tab, h);
  }
  return -1;
}

__device__ int32_t ngram_find(const NgramTableDev &tab, uint64_t packed) {
  const uint64_t h = mix64(packed) & tab.slot_mask;
  return ngram_resolve(tab, packed, h, slot_load(tab, h));
}

__device__ __forceinline__ int key_level(uint64_t key) { return 15 - (int)((key >> 28) & 0xF); }
__device__ __forceinline__ int key_creation(uint64_t key) {
  return 0x0FFFFFFF - (int)(key & 0x0FFFFFFF);
}

// N-gram scores of level L for the nb current beam entries: s_ng[b*k + c] = stored score of
// candidate c among the successors of beam entry b's context, else the miss score.  The
// successor rows are read once, coalesced, all loads independent; each loaded successor is
// compared with the level's k candidates (LDS broadcast reads).  Successor ids are distinct
// within a row and candidate ids within a level, so at most one thread writes a cell.
__device__ __forceinline__ void score_rows(PruneShared &sh, const NgramTableDev &tab, int nb, int k,
                                           int L, int t) {
  const int S = tab.S;
  for (int e = t; e < nb * k; e += PRUNE_THREADS) sh.s_ng[e] = tab.logp_miss;
  __syncthreads();
  for (int idx = t; idx < nb * S; idx += PRUNE_THREADS) {
    const int b = idx / S, j = idx - b * S;
    const int row = sh.beam_row[b];
    if (row >= 0) {
      const int32_t id = tab.succ_ids[(size_t)row * S + j];
      const float lp = tab.succ_logp[(size_t)row * S + j];
      for (int c = 0; c < k; ++c)
        if (sh.cand_id[L * k + c] == id) sh.s_ng[b * k + c] = lp;
    }
  }
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
  if (t == 0) {
    const int prev = ctx_len >= 2 ? ctx_tail[ctx_len - 2] : 0;
    sh.beam_score[0][0] = 0.f;
    sh.beam_tok[0][0] = root;
    sh.beam_prev[0][0] = prev;
    sh.beam_cre[0][0] = -1;                    // the root
    sh.beam_row[0] = ngram_find(tab, pack_context(ctx_len, prev, root));
  }
  int nb = 1, n_best = 0, cur = 0, bcur = 0;
  __syncthreads();
  score_rows(sh, tab, 1, k, 0, t);
  __syncthreads();

  for (int L = 0; L < K; ++L) {
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
      const float s_ng = sh.s_ng[e];
      const float a = __fmul_rn(wl, sh.cand_sc[L * k + c]);
      const float g = __fmul_rn(w_ng, s_ng);
      const float inc = __fmul_rn(__fadd_rn(a, g), wv);
      const float sc = __fadd_rn(sh.beam_score[cur][b], inc);
      tok_out = tok;
      b_out = b;
      return ((uint64_t)f32_sortable(sc) << 32) | ((uint64_t)(15 - L) << 28) |
             (uint64_t)(0x0FFFFFFF - e);
    };

    if (n_new <= PRUNE_FAST * PRUNE_THREADS) {
      // Register-resident path: a thread owns up to two expansions, ranks them by counting
      // the keys that beat them (keys are unique), and -- because it knows the context its
      // expansion would present at the next level -- fetches that context's hash slot
      // already now, so the table probe overlaps with the ranking instead of following it.
      uint64_t key[PRUNE_FAST], packed[PRUNE_FAST], hslot[PRUNE_FAST];
      uint4 raw[PRUNE_FAST];
      int tok[PRUNE_FAST], bb[PRUNE_FAST], rank[PRUNE_FAST];
#pragma unroll
      for (int q = 0; q < PRUNE_FAST; ++q) {
        const int e = t + q * PRUNE_THREADS;
        key[q] = 0;
        if (e < n_new) {
          key[q] = expansion_key(e, tok[q], bb[q]);
          sh.keys[e] = key[q];
          if (!last) {
            packed[q] = pack_context(ctx_len, sh.beam_tok[cur][bb[q]], tok[q]);
            hslot[q] = mix64(packed[q]) & tab.slot_mask;
            raw[q] = slot_load(tab, hslot[q]);
          }
        }
        rank[q] = 0;
      }
      __syncthreads();
      for (int j = 0; j < n_new; ++j) {
        const uint64_t kj = sh.keys[j];
#pragma unroll
        for (int q = 0; q < PRUNE_FAST; ++q) rank[q] += kj > key[q];
      }
#pragma unroll
      for (int q = 0; q < PRUNE_FAST; ++q) {
        const int e = t + q * PRUNE_THREADS;
        if (e < n_new) {
          const int r = rank[q];
          if (r < nb_next) {
            sh.beam_score[nxt][r] = f32_unsortable((uint32_t)(key[q] >> 32));
            sh.beam_tok[nxt][r] = tok[q];
            sh.beam_prev[nxt][r] = sh.beam_tok[cur][bb[q]];
            sh.beam_cre[nxt][r] = e;
          }
          if (r < n_lvl) {
            sh.lvl_key[r] = key[q];
            sh.lvl_tok[r] = tok[q];
            sh.lvl_par[r] = sh.beam_cre[cur][bb[q]];
          }
        }
      }
      // beam_row of this level was last read before the barrier above: safe to overwrite
#pragma unroll
      for (int q = 0; q < PRUNE_FAST; ++q) {
        const int e = t + q * PRUNE_THREADS;
        if (!last && e < n_new && rank[q] < nb_next)
          sh.beam_row[rank[q]] = ngram_resolve(tab, packed[q], hslot[q], raw[q]);
      }
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
          if (!last) row = ngram_find(tab, pack_context(ctx_len, sh.beam_tok[cur][b], tk));
        }
        if (t < n_lvl) {
          sh.lvl_key[t] = kk;
          sh.lvl_tok[t] = tk;
          sh.lvl_par[t] = sh.beam_cre[cur][b];
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
        for (int j = 0; j < n_lvl; ++j) rank += (sh.lvl_key[j] > key);
      } else {
        const int j0 = t - n_best;
        key = sh.lvl_key[j0];
        tok = sh.lvl_tok[j0];
        par = sh.lvl_par[j0];
        rank = j0;
        for (int j = 0; j < n_best; ++j) rank += (sh.best_key[bcur][j] > key);
      }
      if (rank < theta) {
        sh.best_key[bnx][rank] = key;
        sh.best_tok[bnx][rank] = tok;
        sh.best_par[bnx][rank] = par;
      }
    }
    if (!last) score_rows(sh, tab, nb_next, k, L + 1, t);
    n_best = min(theta, n_best + n_lvl);
    bcur = bnx;
    cur = nxt;
    nb = nb_next;
    __syncthreads();
  }

  // emission: root, then level-major; inside a level the best list's order already is
  // (score desc, creation asc)
  const int n_nodes = 1 + n_best;
  if (t < n_best) {
    const int lev = key_level(sh.best_key[bcur][t]);
    int idx = 1;
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
  for (int i = t; i < budget * budget; i += PRUNE_THREADS) mask_out[i] = 0;
  __syncthreads();
  if (t < n_nodes) {
    int j = t;
    for (int hops = 0; j >= 0 && hops <= DART_MAX_K; ++hops) {   // depth <= K: bounded walk
      mask_out[(size_t)t * budget + j] = 1;
      j = sh.out_par[j];
    }
  }
}

hipError_t launch_prune(int batch, const int32_t *ids, const float *scores, int K,
                        const int32_t *ctx_tail, const NgramTableDev &tab,
                        const dart_prune_params &p, const PruneLevelWeights &lw, int32_t *tokens,
                        int32_t *parents, uint8_t *mask, int32_t *n_nodes, hipStream_t st) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void *)prune_kernel,
                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)sizeof(PruneShared));
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(prune_kernel, dim3(batch), dim3(PRUNE_THREADS), sizeof(PruneShared), st, ids,
                     scores, K, ctx_tail, tab, p.k, p.beam_w, p.budget, p.w_ng, lw, tokens, parents,
                     mask, n_nodes);
  return hipGetLastError();
}

}  // namespace dart
