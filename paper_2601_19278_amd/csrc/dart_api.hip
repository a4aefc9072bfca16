// C ABI of the DART drafting step: context creation (weight upload and re-tiling),
// orchestration of the draft forward, top-k, N-gram table build and tree pruning.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <thread>
#include <vector>

#include "dart_internal.h"

using namespace dart;

#define HIP_TRY(expr)                    \
  do {                                   \
    hipError_t e_ = (expr);              \
    if (e_ != hipSuccess) return e_;     \
  } while (0)

namespace dart {

hipError_t raise_dynamic_lds_once(const void *func, int bytes) {
  struct Done {
    const void *func;
    int device;
  };
  static std::mutex lock;
  static std::vector<Done> done;
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  std::lock_guard<std::mutex> hold(lock);
  for (const Done &d : done)
    if (d.func == func && d.device == dev) return hipSuccess;
  HIP_TRY(hipFuncSetAttribute(func, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
  done.push_back(Done{func, dev});
  return hipSuccess;
}

}  // namespace dart

namespace {

size_t elem_size(int dtype) { return dtype == DART_BF16 ? 2 : 4; }

int round_up(int v, int m) { return (v + m - 1) / m * m; }

hipError_t upload(const void *host, size_t bytes, void **dev) {
  HIP_TRY(hipMalloc(dev, bytes));
  return hipMemcpy(*dev, host, bytes, hipMemcpyHostToDevice);
}

// A logical matrix given as a list of row pointers (rows may come from several tensors).
struct RowSource {
  std::vector<const uint8_t *> rows;
  int Kd;
};

// fp32: plain row-major copy.
hipError_t upload_f32(const RowSource &src, DeviceMatrix *out) {
  const int N = (int)src.rows.size();
  std::vector<float> host((size_t)N * src.Kd);
  for (int r = 0; r < N; ++r) memcpy(&host[(size_t)r * src.Kd], src.rows[r], (size_t)src.Kd * 4);
  out->N = out->n_real = N;
  out->Kd = src.Kd;
  return upload(host.data(), host.size() * 4, &out->data);
}

// bf16: re-tile for v_mfma_f32_16x16x32_bf16.  Tile (strip s, k-step t) holds output rows
// 16s..16s+15 and inputs 32t..32t+31; lane l of the consuming wavefront reads the 16 bytes
// at tile + 16*l and must find inputs 32t + 8*(l/16) .. +7 of row 16s + l%16 there (the A
// operand layout of the instruction).  Rows beyond N are zero.
hipError_t upload_bf16_tiles(const RowSource &src, DeviceMatrix *out) {
  const int N = (int)src.rows.size();
  const int strips = (N + 15) / 16, KT = src.Kd / 32;
  const size_t total = (size_t)strips * KT * 512;          // bf16 elements
  uint16_t *host = (uint16_t *)malloc(total * 2);
  if (!host) return hipErrorOutOfMemory;
  auto work = [&](int s0, int s1) {
    for (int s = s0; s < s1; ++s)
      for (int t = 0; t < KT; ++t) {
        uint16_t *tile = host + ((size_t)s * KT + t) * 512;
        for (int l = 0; l < 64; ++l) {
          const int row = s * 16 + (l & 15);
          if (row < N)
            memcpy(tile + l * 8, src.rows[row] + ((size_t)t * 32 + 8 * (l >> 4)) * 2, 16);
          else
            memset(tile + l * 8, 0, 16);
        }
      }
  };
  const int nthr = 8;
  std::vector<std::thread> pool;
  for (int i = 0; i < nthr; ++i)
    pool.emplace_back(work, (int)((int64_t)strips * i / nthr), (int)((int64_t)strips * (i + 1) / nthr));
  for (auto &th : pool) th.join();
  out->N = strips * 16;
  out->n_real = N;
  out->Kd = src.Kd;
  hipError_t e = upload(host, total * 2, &out->data);
  free(host);
  return e;
}

void add_rows(RowSource &src, const void *base, int rows, int Kd, size_t es) {
  for (int r = 0; r < rows; ++r) src.rows.push_back((const uint8_t *)base + (size_t)r * Kd * es);
}

hipError_t upload_matrix(int dtype, const RowSource &src, DeviceMatrix *out) {
  return dtype == DART_BF16 ? upload_bf16_tiles(src, out) : upload_f32(src, out);
}

template <typename T>
hipError_t dev_alloc(T **p, size_t count, bool zero = false) {
  HIP_TRY(hipMalloc((void **)p, count * sizeof(T)));
  if (zero) HIP_TRY(hipMemset(*p, 0, count * sizeof(T)));
  return hipSuccess;
}

hipError_t build(dart_ctx *c, const dart_weights *w) {
  const dart_config &g = c->cfg;
  const size_t es = elem_size(g.dtype);
  const int d = g.d, F = g.ffn, hd = g.head_dim;

  const int in_dim = c->in_dim;            // attention input width: d, or 2d with the front end
  RowSource qkv{{}, in_dim};
  add_rows(qkv, w->wq, c->q_dim, in_dim, es);
  add_rows(qkv, w->wk, c->kv_dim, in_dim, es);
  add_rows(qkv, w->wv, c->kv_dim, in_dim, es);
  HIP_TRY(upload_matrix(g.dtype, qkv, &c->wqkv));

  RowSource wo{{}, c->q_dim};
  add_rows(wo, w->wo, d, c->q_dim, es);
  HIP_TRY(upload_matrix(g.dtype, wo, &c->wo));

  // gate/up: fp32 keeps [gate rows | up rows]; bf16 interleaves groups of four output rows
  // (gate f, gate f+1, up f, up f+1) so that one MFMA lane ends up holding gate/up pairs.
  RowSource gu{{}, d};
  if (g.dtype == DART_BF16) {
    for (int f = 0; f < F; f += 2) {
      gu.rows.push_back((const uint8_t *)w->w_gate + (size_t)f * d * es);
      gu.rows.push_back((const uint8_t *)w->w_gate + (size_t)(f + 1) * d * es);
      gu.rows.push_back((const uint8_t *)w->w_up + (size_t)f * d * es);
      gu.rows.push_back((const uint8_t *)w->w_up + (size_t)(f + 1) * d * es);
    }
  } else {
    add_rows(gu, w->w_gate, F, d, es);
    add_rows(gu, w->w_up, F, d, es);
  }
  HIP_TRY(upload_matrix(g.dtype, gu, &c->wgu));

  RowSource down{{}, F};
  add_rows(down, w->w_down, d, F, es);
  HIP_TRY(upload_matrix(g.dtype, down, &c->wdown));

  RowSource lm{{}, d};
  add_rows(lm, w->w_lm, g.vocab, d, es);
  HIP_TRY(upload_matrix(g.dtype, lm, &c->wlm));

  HIP_TRY(upload(w->w_in_norm, d * es, &c->g_in));
  HIP_TRY(upload(w->w_post_norm, d * es, &c->g_post));
  HIP_TRY(upload(w->w_final_norm, d * es, &c->g_final));
  if (g.qk_norm) {
    HIP_TRY(upload(w->q_norm, hd * es, &c->g_q));
    HIP_TRY(upload(w->k_norm, hd * es, &c->g_k));
  }
  if (g.max_K > 1) HIP_TRY(upload(w->mask_emb, (size_t)(g.max_K - 1) * in_dim * es, &c->mask_emb));
  if (g.front_end) {
    RowSource fc{{}, g.feat_dim};
    add_rows(fc, w->w_fc, d, g.feat_dim, es);
    HIP_TRY(upload_matrix(g.dtype, fc, &c->wfc));
    HIP_TRY(upload(w->embed, (size_t)g.vocab * d * es, &c->embed));
    HIP_TRY(upload(w->w_emb_norm, d * es, &c->g_emb));
  }

  // The batched entry points run every projection on the multi-row kernel, whose matrix pipe
  // would be the co-bound at 128 rows with two-term (hi + lo) bf16 activations.  Their
  // contexts keep an fp16 copy of each matrix (bf16 -> fp16 is exact for 2^-14 <= |w| < 65520)
  // and feed fp16 activations: one product per tile instead of two, and an input rounding of
  // 2^-12 relative, an order of magnitude inside the logit tolerance.
  if (g.dtype == DART_BF16 && g.max_batch > 1) {
    DeviceMatrix *ms[] = {&c->wqkv, &c->wo, &c->wgu, &c->wdown, &c->wlm, &c->wfc};
    for (DeviceMatrix *m : ms) {
      if (!m->data) continue;
      const size_t elems = (size_t)m->N * m->Kd;
      HIP_TRY(hipMalloc(&m->data16, elems * 2));
      HIP_TRY(launch_tiles_to_f16(m->data, m->data16, elems, nullptr));
    }
    HIP_TRY(hipDeviceSynchronize());
  }

  // rotary tables: angle = position * base^(-2i/hd), evaluated in double
  const int half = hd / 2;
  std::vector<float> cs((size_t)c->t_cap * half), sn((size_t)c->t_cap * half);
  for (int i = 0; i < half; ++i) {
    const double inv = std::pow((double)g.rope_base, -2.0 * i / hd);
    for (int p = 0; p < c->t_cap; ++p) {
      cs[(size_t)p * half + i] = (float)std::cos(p * inv);
      sn[(size_t)p * half + i] = (float)std::sin(p * inv);
    }
  }
  HIP_TRY(upload(cs.data(), cs.size() * 4, (void **)&c->rope_cos));
  HIP_TRY(upload(sn.data(), sn.size() * 4, (void **)&c->rope_sin));

  // K/V buffers start zeroed: rows never written must stay finite because the attention
  // kernel multiplies masked keys by probability zero
  const size_t kv_bytes = (size_t)g.max_batch * g.n_kv_heads * c->t_cap * hd * es;
  HIP_TRY(hipMalloc(&c->kbuf, kv_bytes));
  HIP_TRY(hipMemset(c->kbuf, 0, kv_bytes));
  HIP_TRY(hipMalloc(&c->vbuf, kv_bytes));
  HIP_TRY(hipMemset(c->vbuf, 0, kv_bytes));

  const int R = DART_SKINNY_ROWS;
  c->split_qkv = c->split_o = c->split_gu = c->split_down = 1;
  int ch_qkv = 1, ch_o = 1, ch_gu = 1, ch_down = 1;      // k-chunks each projection writes
  c->kv_rows = R;
  if (g.dtype == DART_BF16) {
    c->split_qkv = gemv_bf16_split(in_dim, c->qkv_dim / 16);
    if (g.front_end) c->split_fc = gemv_bf16_split(g.feat_dim, (d + 15) / 16);
    c->split_o = gemv_bf16_split(c->q_dim, (d + 15) / 16);
    c->split_gu = gemv_bf16_split(d, 2 * F / 16);
    c->split_down = gemv_bf16_split(F, (d + 15) / 16);
    ch_qkv = c->split_qkv;
    ch_o = c->split_o;
    ch_gu = c->split_gu;
    ch_down = c->split_down;
    if (g.max_ctx > R && gemv_bf16_row_tiles(in_dim, c->split_qkv) >= 4 &&
        (!g.front_end || gemv_bf16_row_tiles(g.feat_dim, c->split_fc) >= 4))
      c->kv_rows = std::min(1024, round_up(g.max_ctx, 64));
    // the many-row kernel that keeps the skinny kernel's sums takes the whole cold prefix in
    // passes of up to 4096 rows (512 workgroup units: two per compute unit)
    // (with the front end the FC layer goes through the same kernel, in passes of 2048 rows: its
    // fp32 feature rows and their operand tiles are 3d wide)
    c->kv_ordered = g.max_ctx > 32 && gemm_ordered_supported(c->wqkv, c->split_qkv) &&
                    (!g.front_end || gemm_ordered_supported(c->wfc, c->split_fc));
    if (c->kv_ordered) c->kv_rows = std::min(g.front_end ? 2048 : 4096, round_up(g.max_ctx, 64));
    if (g.max_batch > 1) {     // the batched entry point runs on the multi-row kernel
      c->gch_qkv = gemm_bf16_chunks(in_dim, c->qkv_dim / 16);
      c->gch_o = gemm_bf16_chunks(c->q_dim, (d + 15) / 16);
      c->gch_gu = gemm_bf16_chunks(d, 2 * F / 16);
      c->gch_down = gemm_bf16_chunks(F, (d + 15) / 16);
      if (g.front_end) c->gch_fc = gemm_bf16_chunks(g.feat_dim, (d + 15) / 16);
      ch_qkv = std::max(ch_qkv, c->gch_qkv);
      ch_o = std::max(ch_o, c->gch_o);
      ch_gu = std::max(ch_gu, c->gch_gu);
      ch_down = std::max(ch_down, c->gch_down);
      c->kv_rows = std::max(c->kv_rows, std::min(1024, round_up(g.max_ctx, 64)));
    }
  }
  // one pass carries the query rows of up to DART_SEQ_GROUP sequences
  c->ws_rows = std::max(R, std::min(g.max_batch, DART_SEQ_GROUP) * g.max_K);
  const size_t W = c->ws_rows;
  // attention partials: per query vector, at most one per 128-key split (the key sub-ranges of
  // a split are merged inside the attention kernel)
  c->max_splits = c->t_cap / ATTN_KEY_CHUNK;
  const int att_rows = g.max_K;
  const size_t att_slots = (size_t)std::min(g.max_batch, DART_SEQ_GROUP) * att_rows * g.n_q_heads *
                           c->max_splits;
  const size_t proj_elems = std::max(std::max((size_t)ch_o * d, (size_t)ch_down * d),
                                     (size_t)ch_gu * 2 * F);
  HIP_TRY(dev_alloc(&c->xn, W * in_dim));
  HIP_TRY(dev_alloc(&c->resid, W * d));
  HIP_TRY(dev_alloc(&c->qkv, (size_t)ch_qkv * W * c->qkv_dim));
  HIP_TRY(hipMalloc(&c->qrot, W * c->q_dim * 4));
  HIP_TRY(dev_alloc(&c->att_part, att_slots * hd));
  HIP_TRY(dev_alloc(&c->att_ml, att_slots * 2));
  HIP_TRY(dev_alloc(&c->att_out, W * c->q_dim));
  HIP_TRY(dev_alloc(&c->proj, W * proj_elems));
  HIP_TRY(dev_alloc(&c->y, W * d));
  HIP_TRY(dev_alloc(&c->yn, W * d));
  HIP_TRY(dev_alloc(&c->hmid, W * F));
  HIP_TRY(dev_alloc(&c->u, W * d));
  if (g.dtype == DART_BF16) {
    size_t pb = gemm_bf16_pack_bytes(c->kv_rows, in_dim);
    for (int kd : {in_dim, c->q_dim, F}) pb = std::max(pb, gemm_bf16_pack_bytes(c->ws_rows, kd));
    if (g.front_end)
      pb = std::max(pb, gemm_bf16_pack_bytes(std::max(c->ws_rows, c->kv_rows), g.feat_dim));
    HIP_TRY(hipMalloc(&c->xpack, pb));
    if (g.max_batch > 1) HIP_TRY(hipMalloc(&c->xpack2, gemm_bf16_pack_bytes(c->ws_rows, F)));
  }
  HIP_TRY(dev_alloc(&c->xn_kv, (size_t)c->kv_rows * in_dim));
  if (g.front_end) {
    c->fc_rows = std::max(c->ws_rows, c->kv_rows);
    const int ch_fc = g.dtype == DART_BF16 ? std::max(c->split_fc, c->gch_fc) : 1;
    HIP_TRY(dev_alloc(&c->feat32, (size_t)c->fc_rows * g.feat_dim));
    HIP_TRY(dev_alloc(&c->fc_part, (size_t)ch_fc * c->fc_rows * d));
  }
  HIP_TRY(dev_alloc(&c->kv_part, (size_t)ch_qkv * c->kv_rows * 2 * c->kv_dim));

  if (g.dtype == DART_BF16 && gemv_bf16_chunks(d) > 1) {
    c->split_lm = gemv_bf16_chunks(d);
    c->lm_stride = (size_t)round_up(g.vocab, 16);
    HIP_TRY(dev_alloc(&c->lm_part, (size_t)c->split_lm * R * c->lm_stride));
  }
  c->max_rows = g.max_batch * g.max_K;
  c->topk_chunks_max = topk_chunks(g.vocab);
  if (g.dtype == DART_BF16)
    c->lm_select_wgs = gemv_bf16_select_wgs(c->wlm, (g.vocab + 15) / 16, std::min(g.max_K, 8));
  c->topk_chunks_max = std::max(c->topk_chunks_max, c->lm_select_wgs);
  // logits of one group of sequences, for the combined calls when the caller passes no buffer
  const int tmp_rows = std::min(c->max_rows, DART_SEQ_GROUP * g.max_K);
  HIP_TRY(dev_alloc(&c->logits_tmp, (size_t)tmp_rows * g.vocab));
  HIP_TRY(dev_alloc(&c->topk_cand, (size_t)c->max_rows * c->topk_chunks_max * DART_MAX_TOPK));
  HIP_TRY(dev_alloc(&c->topk_ms, (size_t)c->max_rows * c->topk_chunks_max * 2));
  return hipSuccess;
}

dart_status from_hip(hipError_t e) {
  if (e == hipSuccess) return DART_OK;
  return e == hipErrorOutOfMemory ? DART_ERR_OOM : DART_ERR_HIP;
}

// Projection of M rows of X (fp32 [M][W.Kd]) through output rows [row0, row0+nrows) of W;
// out[chunk][m][j] with row stride out_stride and chunk stride chunk_stride.
// split: k-chunks of the matrix on the skinny kernel (fixed per matrix at create time so that
// every call cuts k the same way; 1 where the output must be complete in one chunk).
// gch > 0: take the multi-row kernel with gch k-chunks (the batched entry point).
hipError_t project(const dart_ctx *c, const DeviceMatrix &W, int row0, int nrows, const float *X,
                   int M, float *out, int out_stride, size_t chunk_stride, int split, int gch,
                   int *chunks, hipStream_t st) {
  const int R = DART_SKINNY_ROWS;
  if (c->cfg.dtype == DART_BF16 && gch > 0) {
    *chunks = gch;
    return launch_gemm_bf16(W, row0 / 16, (nrows + 15) / 16, X, M, c->xpack, out, out_stride,
                            chunk_stride, gch, 0, st);
  }
  if (c->cfg.dtype == DART_BF16) {
    if (M <= R || gemv_bf16_row_tiles(W.Kd, split) >= 2)
      return launch_gemv_bf16(W, row0 / 16, (nrows + 15) / 16, X, M, out, out_stride, chunk_stride,
                              split, chunks, st);
    for (int m0 = 0; m0 < M; m0 += R)
      HIP_TRY(launch_gemv_bf16(W, row0 / 16, (nrows + 15) / 16, X + (size_t)m0 * W.Kd,
                               std::min(R, M - m0), out + (size_t)m0 * out_stride, out_stride,
                               chunk_stride, split, chunks, st));
    return hipSuccess;
  }
  *chunks = 1;
  for (int m0 = 0; m0 < M; m0 += R)
    HIP_TRY(launch_gemv_f32(W, row0, nrows, X + (size_t)m0 * W.Kd, std::min(R, M - m0),
                            out + (size_t)m0 * out_stride, out_stride, st));
  return hipSuccess;
}

// LM head (Sec. 3.2) on the final-normed rows X (null on the multi-row path: operand tiles
// already packed).  The skinny kernel writes the caller's logits directly when d fits one
// k-chunk; a longer d goes through chunk partials and one more pass that adds them.
// Candidate extraction fused into the LM head (dart_draft_forward_topk): k, eps and outputs.
struct FusedCand {
  int k;
  float eps;
  int32_t *ids;
  float *scores;
};

hipError_t lm_head(const dart_ctx *c, const float *X, int rows, bool gemm, float *logits,
                   hipStream_t st, const FusedCand *fc = nullptr) {
  const int V = c->cfg.vocab;
  int chunks = 1;
  if (fc) {
    // the LM-head workgroups select their own candidates; the row merge finishes (Alg. 1, App. D)
    const GemvTopk tk{c->topk_cand, c->topk_ms, fc->k};
    HIP_TRY(launch_gemv_bf16(c->wlm, 0, (V + 15) / 16, X, rows, logits, V, 0, 1, &chunks, st, &tk));
    return launch_topk_merge(c->topk_cand, c->topk_ms, rows, fc->k, c->lm_select_wgs, fc->eps, fc->ids,
                             fc->scores, st);
  }
  if (gemm || c->split_lm == 1 || c->cfg.dtype != DART_BF16)
    return project(c, c->wlm, 0, V, X, rows, logits, V, 0, 1, gemm ? 1 : 0, &chunks, st);
  const size_t cs = (size_t)DART_SKINNY_ROWS * c->lm_stride;
  for (int m0 = 0; m0 < rows; m0 += DART_SKINNY_ROWS) {
    const int m = std::min(DART_SKINNY_ROWS, rows - m0);
    HIP_TRY(launch_gemv_bf16(c->wlm, 0, (V + 15) / 16, X + (size_t)m0 * c->cfg.d, m, c->lm_part,
                             (int)c->lm_stride, cs, c->split_lm, &chunks, st));
    HIP_TRY(launch_sum_chunks(c->lm_part, chunks, cs, (int)c->lm_stride, m, V,
                              logits + (size_t)m0 * V, V, st));
  }
  return hipSuccess;
}

// One sequence of a forward call.
struct SeqJob {
  int slot;
  const void *hidden;          // prefix representation, or the feature rows with the front end
  int n, n_cached;
  const int32_t *tokens = nullptr;   // front end: token following each position
};

// Layer input of the rows of a pass: xn = normed attention input ([rows][in_dim]), resid = raw
// residual rows of the query rows (may be null for a K/V-only pass).  Without the front end
// the rows are gathered from the prefix representation / mask embeddings and normed; with it
// (Sec. 3.2) the feature rows first go through the FC layer and are joined by the shifted
// token embeddings.
hipError_t input_stage(dart_ctx *c, const SeqBatch &sb, float *xn, float *resid, bool gemm,
                       hipStream_t st) {
  const dart_config &g = c->cfg;
  if (!g.front_end)
    return launch_rmsnorm_gather(g.dtype, sb, c->mask_emb, c->g_in, g.d, g.rms_eps, xn, resid,
                                 gemm ? c->xpack : nullptr, gemm_bf16_terms(c->wqkv), st);
  const int M = sb.row_off[sb.B];
  HIP_TRY(launch_feature_rows(g.dtype, sb, g.feat_dim, c->feat32, st));
  const size_t cs = (size_t)c->fc_rows * g.d;
  int chunks = 1;
  HIP_TRY(project(c, c->wfc, 0, g.d, c->feat32, M, c->fc_part, g.d, cs, c->split_fc,
                  gemm ? c->gch_fc : 0, &chunks, st));
  return launch_front_norm(g.dtype, sb, c->fc_part, chunks, cs, c->embed, c->mask_emb, c->g_in,
                           c->g_emb, g.d, g.rms_eps, xn, resid, st);
}

// K/V-only pass: norm + K and V projection + append for the rows described by sb (sb.K = 0,
// at most kv_rows rows).
hipError_t kv_pass(dart_ctx *c, const SeqBatch &sb, bool gemm, hipStream_t st) {
  const dart_config &g = c->cfg;
  const int M = sb.row_off[sb.B];
  if (!gemm && c->kv_ordered && M > 32 && g.front_end) {
    // single-sequence call with the front end, many rows: the FC layer and the K/V projection both
    // run on the order-preserving many-row kernel (the skinny kernel's sums bit for bit, chunk
    // partials already added), their fp32 inputs packed as two-term operand tiles in between
    HIP_TRY(launch_feature_rows(g.dtype, sb, g.feat_dim, c->feat32, st));
    HIP_TRY(launch_pack_rows(c->feat32, M, g.feat_dim, 2, c->xpack, st));
    HIP_TRY(launch_gemm_ordered(c->wfc, 0, (g.d + 15) / 16, M, c->xpack, c->fc_part, g.d, c->split_fc, st));
    HIP_TRY(launch_front_norm(g.dtype, sb, c->fc_part, 1, 0, c->embed, c->mask_emb, c->g_in, c->g_emb, g.d,
                              g.rms_eps, c->xn_kv, nullptr, st));
    HIP_TRY(launch_pack_rows(c->xn_kv, M, c->in_dim, 2, c->xpack, st));
    HIP_TRY(launch_gemm_ordered(c->wqkv, c->q_dim / 16, 2 * c->kv_dim / 16, M, c->xpack, c->kv_part,
                                2 * c->kv_dim, c->split_qkv, st));
    return launch_qkv_post(c, sb, c->kv_part, 1, 0, 2 * c->kv_dim, c->q_dim, st);
  }
  if (!gemm && c->kv_ordered && M > 32) {
    // single-sequence call, many rows: the input norm writes two-term operand tiles, the
    // order-preserving many-row kernel gives the skinny kernel's K/V sums bit for bit
    HIP_TRY(launch_norm_pack_rows(sb, c->mask_emb, c->g_in, g.d, g.rms_eps, c->xn_kv, c->xpack, st));
    HIP_TRY(launch_gemm_ordered(c->wqkv, c->q_dim / 16, 2 * c->kv_dim / 16, M, c->xpack, c->kv_part,
                                2 * c->kv_dim, c->split_qkv, st));
    return launch_qkv_post(c, sb, c->kv_part, 1, 0, 2 * c->kv_dim, c->q_dim, st);
  }
  HIP_TRY(input_stage(c, sb, c->xn_kv, nullptr, gemm, st));
  const size_t cs = (size_t)c->kv_rows * 2 * c->kv_dim;
  int chunks = 1;
  const float *xin = gemm && !g.front_end ? nullptr : c->xn_kv;    // null: operand tiles already packed
  HIP_TRY(project(c, c->wqkv, c->q_dim, 2 * c->kv_dim, xin, M, c->kv_part, 2 * c->kv_dim, cs,
                  c->split_qkv, gemm ? c->gch_qkv : 0, &chunks, st));
  return launch_qkv_post(c, sb, c->kv_part, chunks, cs, 2 * c->kv_dim, c->q_dim, st);
}

// Draft forward of up to DART_SEQ_GROUP sequences; logits [B][K][vocab].
// gemm: every projection runs on the multi-row kernel (the batched entry point on bf16
// weights).  The two kernels add a row's products in different orders, so a K/V slot filled
// through one entry point is reused by the other only to rounding, not bit for bit.
hipError_t forward_group(dart_ctx *c, int B, const SeqJob *jobs, int K, bool gemm, float *logits,
                         hipStream_t st, const FusedCand *fc = nullptr) {
  const dart_config &g = c->cfg;
  const int R = DART_SKINNY_ROWS;
  gemm = gemm && g.dtype == DART_BF16;
  // A single sequence with few new rows takes one pass for all of them; otherwise the prefix
  // rows that are not query rows go through K/V-only passes first.
  const bool combined = !gemm && B == 1 && (jobs[0].n - jobs[0].n_cached) + K - 1 <= R;
  if (!combined) {
    SeqBatch sb{};
    auto flush = [&]() -> hipError_t {
      if (sb.B == 0) return hipSuccess;
      hipError_t e = kv_pass(c, sb, gemm, st);
      sb = SeqBatch{};
      return e;
    };
    for (int b = 0; b < B; ++b) {
      int r0 = jobs[b].n_cached;
      while (r0 < jobs[b].n - 1) {
        const int room = c->kv_rows - sb.row_off[sb.B];
        const int take = std::min(room, jobs[b].n - 1 - r0);
        const int i = sb.B++;
        sb.hidden[i] = jobs[b].hidden;
        sb.tokens[i] = jobs[b].tokens;
        sb.n[i] = jobs[b].n;
        sb.pos0[i] = r0;
        sb.slot[i] = jobs[b].slot;
        sb.row_off[i + 1] = sb.row_off[i] + take;
        r0 += take;
        if (sb.row_off[sb.B] == c->kv_rows || sb.B == DART_SEQ_GROUP) HIP_TRY(flush());
      }
    }
    HIP_TRY(flush());
  }

  SeqBatch sb{};
  sb.B = B;
  sb.K = K;
  for (int b = 0; b < B; ++b) {
    sb.hidden[b] = jobs[b].hidden;
    sb.tokens[b] = jobs[b].tokens;
    sb.n[b] = jobs[b].n;
    sb.pos0[b] = combined ? jobs[b].n_cached : jobs[b].n - 1;
    sb.slot[b] = jobs[b].slot;
    sb.row_off[b + 1] = sb.row_off[b] + (jobs[b].n - sb.pos0[b]) + K - 1;
  }
  const int M = sb.row_off[B], QR = B * K;       // pass rows, query rows
  const size_t W = c->ws_rows;
  HIP_TRY(input_stage(c, sb, c->xn, c->resid, gemm, st));
  int chunks = 1;
  size_t cs = W * c->qkv_dim;
  HIP_TRY(project(c, c->wqkv, 0, c->qkv_dim, gemm && !g.front_end ? nullptr : c->xn, M, c->qkv,
                  c->qkv_dim, cs, c->split_qkv,
                  gemm ? c->gch_qkv : 0, &chunks, st));
  HIP_TRY(launch_qkv_post(c, sb, c->qkv, chunks, cs, c->qkv_dim, 0, st));
  // (an odd number of 32-input steps would need a zeroed extra step in the packed operand)
  const bool pack_att = gemm && (c->q_dim / 32) % 2 == 0;
  HIP_TRY(launch_attention(c, sb, pack_att ? c->xpack : nullptr, gemm_bf16_terms(c->wo), st));

  cs = W * g.d;
  HIP_TRY(project(c, c->wo, 0, g.d, pack_att ? nullptr : c->att_out, QR, c->proj, g.d, cs, c->split_o,
                  gemm ? c->gch_o : 0, &chunks, st));
  // on the multi-row path the norm kernels write the next projection's operand tiles themselves
  HIP_TRY(launch_resid_norm(g.dtype, c->resid, c->proj, chunks, cs, g.d, c->g_post, QR, g.d,
                            g.rms_eps, c->y, gemm ? nullptr : c->yn, gemm ? c->xpack : nullptr,
                            gemm_bf16_terms(c->wgu), st));
  const float *yn_in = gemm ? nullptr : c->yn;
  cs = W * 2 * g.ffn;
  // SwiGLU in the gate/up projection's epilogue when its k range is not cut; with fp16 operands
  // the epilogue writes the down projection's operand tiles itself (no fp32 round trip, no
  // conversion pass; an odd number of 32-input steps would need a zeroed extra step)
  const bool fuse_act = gemm && c->gch_gu == 1;
  const bool fuse_pack = fuse_act && c->xpack2 && gemm_bf16_terms(c->wdown) == 1 && (g.ffn / 32) % 2 == 0;
  if (fuse_act) {
    HIP_TRY(launch_gemm_bf16(c->wgu, 0, 2 * g.ffn / 16, yn_in, QR, c->xpack, c->hmid, g.ffn, 0, 1,
                             fuse_pack ? 2 : 1, st, c->xpack2));
  } else {
    HIP_TRY(project(c, c->wgu, 0, 2 * g.ffn, yn_in, QR, c->proj, 2 * g.ffn, cs, c->split_gu,
                    gemm ? c->gch_gu : 0, &chunks, st));
    HIP_TRY(launch_swiglu(c->proj, chunks, cs, QR, g.ffn, g.dtype == DART_BF16, c->hmid, st));
  }
  cs = W * g.d;
  if (fuse_pack) {
    chunks = c->gch_down;
    HIP_TRY(launch_gemm_bf16(c->wdown, 0, (g.d + 15) / 16, nullptr, QR, c->xpack2, c->proj, g.d, cs,
                             chunks, 0, st));
  } else {
    HIP_TRY(project(c, c->wdown, 0, g.d, c->hmid, QR, c->proj, g.d, cs, c->split_down,
                    gemm ? c->gch_down : 0, &chunks, st));
  }
  HIP_TRY(launch_resid_norm(g.dtype, c->y, c->proj, chunks, cs, g.d, c->g_final, QR, g.d, g.rms_eps,
                            gemm ? nullptr : c->u, gemm ? nullptr : c->yn, gemm ? c->xpack : nullptr,
                            gemm_bf16_terms(c->wlm), st));
  return lm_head(c, yn_in, QR, gemm, logits, st, fc);
}

dart_status check_forward_args(const dart_ctx *c, int seq, const void *hidden, int n, int n_cached,
                               int K, const float *logits) {
  if (!c || !hidden || !logits) return DART_ERR_ARG;
  if (seq < 0 || seq >= c->cfg.max_batch || K < 1 || K > c->cfg.max_K || n < 1 || n_cached < 0)
    return DART_ERR_ARG;
  if (n > c->cfg.max_ctx) return DART_ERR_SHAPE;
  if (n_cached > n - 1 || n_cached > c->cached_rows[seq]) return DART_ERR_STATE;
  return DART_OK;
}

}  // namespace

extern "C" {

const char *dart_status_str(dart_status s) {
  switch (s) {
    case DART_OK: return "ok";
    case DART_ERR_ARG: return "invalid argument";
    case DART_ERR_SHAPE: return "shape mismatch";
    case DART_ERR_OOM: return "out of memory";
    case DART_ERR_HIP: return "HIP runtime error";
    case DART_ERR_STATE: return "invalid call sequence";
  }
  return "unknown status";
}

dart_status dart_create(const dart_config *cfg, const dart_weights *w, dart_ctx **out) {
  if (!cfg || !w || !out) return DART_ERR_ARG;
  *out = nullptr;
  const dart_config &g = *cfg;
  if (g.d < 1 || g.n_q_heads < 1 || g.n_kv_heads < 1 || g.ffn < 1 || g.vocab < 1 || g.max_ctx < 1 ||
      g.max_K < 1 || g.max_K > DART_MAX_K || g.max_batch < 1)
    return DART_ERR_ARG;
  if (g.head_dim != 64 && g.head_dim != 128) return DART_ERR_ARG;
  if (g.n_q_heads % g.n_kv_heads != 0 || g.n_q_heads / g.n_kv_heads > 8) return DART_ERR_ARG;
  if (g.dtype != DART_F32 && g.dtype != DART_BF16) return DART_ERR_ARG;
  const int q_dim = g.n_q_heads * g.head_dim;
  if (g.front_end != 0 && g.front_end != 1) return DART_ERR_ARG;
  if (g.front_end) {
    if (g.feat_dim < 8 || g.feat_dim > 16384 || g.feat_dim % (g.dtype == DART_BF16 ? 32 : 8) ||
        2 * g.d > 16384)
      return DART_ERR_ARG;
    if (!w->w_fc || !w->embed || !w->w_emb_norm) return DART_ERR_ARG;
  }
  if (g.dtype == DART_BF16) {
    if (g.d % 32 || q_dim % 32 || g.ffn % 32) return DART_ERR_ARG;
  } else if (g.d % 8 || g.ffn % 4) {
    return DART_ERR_ARG;
  }
  if (g.d > 16384) return DART_ERR_ARG;
  if (g.max_ctx + g.max_K > 32768) return DART_ERR_ARG;   // at most 256 key splits of 128
  if (!w->w_in_norm || !w->wq || !w->wk || !w->wv || !w->wo || !w->w_post_norm || !w->w_gate ||
      !w->w_up || !w->w_down || !w->w_final_norm || !w->w_lm)
    return DART_ERR_ARG;
  if (g.qk_norm && (!w->q_norm || !w->k_norm)) return DART_ERR_ARG;
  if (g.max_K > 1 && !w->mask_emb) return DART_ERR_ARG;

  dart_ctx *c = new (std::nothrow) dart_ctx();
  if (!c) return DART_ERR_OOM;
  c->cfg = g;
  c->in_dim = g.front_end ? 2 * g.d : g.d;
  c->q_dim = q_dim;
  c->kv_dim = g.n_kv_heads * g.head_dim;
  c->qkv_dim = c->q_dim + 2 * c->kv_dim;
  c->t_cap = round_up(g.max_ctx + g.max_K - 1, ATTN_KEY_CHUNK);   // whole key chunks per row
  c->cached_rows = (int *)calloc(g.max_batch, sizeof(int));
  if (!c->cached_rows) {
    delete c;
    return DART_ERR_OOM;
  }
  hipError_t e = build(c, w);
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) {
    (void)hipGetLastError();
    dart_destroy(c);
    return from_hip(e);
  }
  *out = c;
  return DART_OK;
}

void dart_destroy(dart_ctx *c) {
  if (!c) return;
  void *bufs[] = {c->wqkv.data16, c->wo.data16, c->wgu.data16, c->wdown.data16, c->wlm.data16,
                  c->wfc.data16,
                  c->wqkv.data, c->wo.data, c->wgu.data, c->wdown.data, c->wlm.data, c->g_in,
                  c->g_post, c->g_final, c->g_q, c->g_k, c->mask_emb, c->rope_cos, c->rope_sin,
                  c->kbuf, c->vbuf, c->xn, c->resid, c->qkv, c->qrot, c->att_part, c->att_ml,
                  c->att_out, c->proj, c->y, c->yn, c->hmid, c->u, c->topk_cand, c->topk_ms,
                  c->xn_kv, c->kv_part, c->lm_part, c->logits_tmp, c->xpack, c->xpack2, c->wfc.data, c->embed, c->g_emb, c->feat32,
                  c->fc_part};
  for (void *p : bufs)
    if (p) (void)hipFree(p);
  free(c->cached_rows);
  delete c;
}

dart_status dart_reset(dart_ctx *c, int seq) {
  if (!c || seq < 0 || seq >= c->cfg.max_batch) return DART_ERR_ARG;
  c->cached_rows[seq] = 0;
  return DART_OK;
}

dart_status dart_draft_forward_features(dart_ctx *c, int seq, const void *features,
                                        const int32_t *next_tokens, int ctx_len, int n_cached,
                                        int K, float *logits_out, void *stream) {
  dart_status s = check_forward_args(c, seq, features, ctx_len, n_cached, K, logits_out);
  if (s != DART_OK) return s;
  if (!next_tokens) return DART_ERR_ARG;
  if (!c->cfg.front_end) return DART_ERR_STATE;
  SeqJob job{seq, features, ctx_len, n_cached};
  job.tokens = next_tokens;
  c->cached_rows[seq] = 0;           // a failed launch sequence leaves the slot undefined
  hipError_t e = forward_group(c, 1, &job, K, false, logits_out, (hipStream_t)stream);
  if (e != hipSuccess) return from_hip(e);
  c->cached_rows[seq] = ctx_len;
  return DART_OK;
}

dart_status dart_draft_forward(dart_ctx *c, int seq, const void *hidden, int ctx_len, int n_cached,
                               int K, float *logits_out, void *stream) {
  dart_status s = check_forward_args(c, seq, hidden, ctx_len, n_cached, K, logits_out);
  if (s != DART_OK) return s;
  if (c->cfg.front_end) return DART_ERR_STATE;
  const SeqJob job{seq, hidden, ctx_len, n_cached};
  c->cached_rows[seq] = 0;           // a failed launch sequence leaves the slot undefined
  hipError_t e = forward_group(c, 1, &job, K, false, logits_out, (hipStream_t)stream);
  if (e != hipSuccess) return from_hip(e);
  c->cached_rows[seq] = ctx_len;
  return DART_OK;
}

// Shared body of the two single-sequence combined calls (the job carries tokens with the front end).
static dart_status forward_topk_one(dart_ctx *c, const SeqJob &job, int K, int k, float eps,
                                    float *logits_out, int32_t *ids_out, float *scores_out, void *stream) {
  if (!ids_out || !scores_out) return DART_ERR_ARG;
  if (k < 1 || k > DART_MAX_TOPK || k > c->cfg.vocab) return DART_ERR_ARG;
  c->cached_rows[job.slot] = 0;      // a failed launch sequence leaves the slot undefined
  hipError_t e;
  if (c->lm_select_wgs > 0 && K <= 8) {
    const FusedCand fc{k, eps, ids_out, scores_out};
    e = forward_group(c, 1, &job, K, false, logits_out, (hipStream_t)stream, &fc);
  } else {
    // shapes the fused selection does not serve (fp32 storage, more than 8 rows, a d longer than
    // one k-chunk): the two steps one after the other, same results
    float *logits = logits_out ? logits_out : c->logits_tmp;
    e = forward_group(c, 1, &job, K, false, logits, (hipStream_t)stream);
    if (e == hipSuccess)
      e = launch_topk(c, logits, K, c->cfg.vocab, k, eps, ids_out, scores_out, (hipStream_t)stream);
  }
  if (e != hipSuccess) return from_hip(e);
  c->cached_rows[job.slot] = job.n;
  return DART_OK;
}

dart_status dart_draft_forward_topk(dart_ctx *c, int seq, const void *hidden, int ctx_len, int n_cached,
                                    int K, int k, float eps, float *logits_out, int32_t *ids_out,
                                    float *scores_out, void *stream) {
  float dummy = 0.f;
  dart_status s = check_forward_args(c, seq, hidden, ctx_len, n_cached, K, &dummy);
  if (s != DART_OK) return s;
  if (c->cfg.front_end) return DART_ERR_STATE;
  const SeqJob job{seq, hidden, ctx_len, n_cached};
  return forward_topk_one(c, job, K, k, eps, logits_out, ids_out, scores_out, stream);
}

dart_status dart_draft_forward_features_topk(dart_ctx *c, int seq, const void *features,
                                             const int32_t *next_tokens, int ctx_len, int n_cached,
                                             int K, int k, float eps, float *logits_out,
                                             int32_t *ids_out, float *scores_out, void *stream) {
  float dummy = 0.f;
  dart_status s = check_forward_args(c, seq, features, ctx_len, n_cached, K, &dummy);
  if (s != DART_OK) return s;
  if (!next_tokens) return DART_ERR_ARG;
  if (!c->cfg.front_end) return DART_ERR_STATE;
  SeqJob job{seq, features, ctx_len, n_cached};
  job.tokens = next_tokens;
  return forward_topk_one(c, job, K, k, eps, logits_out, ids_out, scores_out, stream);
}

// Shared body of the two batched entry points (tokens = null without the front end).
static dart_status forward_batched(dart_ctx *c, int batch, const void *const *rows,
                                   const int32_t *const *tokens, const int32_t *ctx_len,
                                   const int32_t *n_cached, int K, float *logits_out, void *stream) {
  if (!c || !rows || !ctx_len || !n_cached || !logits_out) return DART_ERR_ARG;
  if (batch < 1 || batch > c->cfg.max_batch) return DART_ERR_ARG;
  if ((c->cfg.front_end != 0) != (tokens != nullptr)) return DART_ERR_STATE;
  for (int b = 0; b < batch; ++b) {
    dart_status s = check_forward_args(c, b, rows[b], ctx_len[b], n_cached[b], K, logits_out);
    if (s != DART_OK) return s;
    if (tokens && !tokens[b]) return DART_ERR_ARG;
  }
  for (int b0 = 0; b0 < batch; b0 += DART_SEQ_GROUP) {
    const int nb = std::min(DART_SEQ_GROUP, batch - b0);
    SeqJob jobs[DART_SEQ_GROUP];
    for (int i = 0; i < nb; ++i) {
      jobs[i] = SeqJob{b0 + i, rows[b0 + i], ctx_len[b0 + i], n_cached[b0 + i]};
      if (tokens) jobs[i].tokens = tokens[b0 + i];
      c->cached_rows[b0 + i] = 0;
    }
    hipError_t e = forward_group(c, nb, jobs, K, true, logits_out + (size_t)b0 * K * c->cfg.vocab,
                                 (hipStream_t)stream);
    if (e != hipSuccess) return from_hip(e);
    for (int i = 0; i < nb; ++i) c->cached_rows[b0 + i] = ctx_len[b0 + i];
  }
  return DART_OK;
}

dart_status dart_draft_forward_topk_batched(dart_ctx *c, int batch, const void *const *hidden,
                                            const int32_t *ctx_len, const int32_t *n_cached, int K,
                                            int k, float eps, float *logits_out, int32_t *ids_out,
                                            float *scores_out, void *stream) {
  if (!c || !hidden || !ctx_len || !n_cached || !ids_out || !scores_out) return DART_ERR_ARG;
  if (batch < 1 || batch > c->cfg.max_batch) return DART_ERR_ARG;
  if (c->cfg.front_end) return DART_ERR_STATE;
  float dummy = 0.f;
  for (int b = 0; b < batch; ++b) {
    dart_status s = check_forward_args(c, b, hidden[b], ctx_len[b], n_cached[b], K, &dummy);
    if (s != DART_OK) return s;
  }
  if (k < 1 || k > DART_MAX_TOPK || k > c->cfg.vocab) return DART_ERR_ARG;
  const int V = c->cfg.vocab;
  hipStream_t st = (hipStream_t)stream;
  for (int b0 = 0; b0 < batch; b0 += DART_SEQ_GROUP) {
    const int nb = std::min(DART_SEQ_GROUP, batch - b0);
    SeqJob jobs[DART_SEQ_GROUP];
    for (int i = 0; i < nb; ++i) {
      jobs[i] = SeqJob{b0 + i, hidden[b0 + i], ctx_len[b0 + i], n_cached[b0 + i]};
      c->cached_rows[b0 + i] = 0;
    }
    float *lg = logits_out ? logits_out + (size_t)b0 * K * V : nullptr;
    int32_t *ids = ids_out + (size_t)b0 * K * k;
    float *sc = scores_out + (size_t)b0 * K * k;
    // The multi-row LM head leaves the selection to the top-k kernels: a form of it whose
    // workgroups select their rows' candidates in the epilogue was built and measured no faster
    // (the selection is bound by instruction issue, about 25 instructions per logit in either
    // place, and inside the LM head nothing overlaps it).
    if (!lg) lg = c->logits_tmp;
    hipError_t e = forward_group(c, nb, jobs, K, true, lg, st);
    if (e == hipSuccess) e = launch_topk(c, lg, nb * K, V, k, eps, ids, sc, st);
    if (e != hipSuccess) return from_hip(e);
    for (int i = 0; i < nb; ++i) c->cached_rows[b0 + i] = ctx_len[b0 + i];
  }
  return DART_OK;
}

dart_status dart_draft_forward_batched(dart_ctx *c, int batch, const void *const *hidden,
                                       const int32_t *ctx_len, const int32_t *n_cached, int K,
                                       float *logits_out, void *stream) {
  return forward_batched(c, batch, hidden, nullptr, ctx_len, n_cached, K, logits_out, stream);
}

dart_status dart_draft_forward_features_batched(dart_ctx *c, int batch, const void *const *features,
                                                const int32_t *const *next_tokens,
                                                const int32_t *ctx_len, const int32_t *n_cached,
                                                int K, float *logits_out, void *stream) {
  if (!next_tokens) return DART_ERR_ARG;
  return forward_batched(c, batch, features, next_tokens, ctx_len, n_cached, K, logits_out, stream);
}

dart_status dart_topk(dart_ctx *c, const float *logits, int rows, int vocab, int k, float eps,
                      int32_t *ids_out, float *scores_out, void *stream) {
  if (!c || !logits || !ids_out || !scores_out) return DART_ERR_ARG;
  if (rows < 1 || vocab < 1 || k < 1 || k > DART_MAX_TOPK || k > vocab) return DART_ERR_ARG;
  if (vocab > c->cfg.vocab || rows > c->max_rows) return DART_ERR_SHAPE;
  return from_hip(launch_topk(c, logits, rows, vocab, k, eps, ids_out, scores_out,
                              (hipStream_t)stream));
}

// Host arrays of one hashed table -> device.  ctx_len tokens per context; stored score of a
// successor = min(0, log(scale * count / sum(row counts) + eps)) in fp64, rounded once.
static dart_status build_table(int ctx_len, int64_t n_keys, int S, const int32_t *keys,
                               const int32_t *succ_ids, const int32_t *succ_counts, double eps_d,
                               double scale, void **d_slots, void **d_ids, void **d_logp,
                               uint64_t *slot_mask, float *miss_out) {
  for (int64_t i = 0; i < n_keys * ctx_len; ++i)
    if (keys[i] < 0) return DART_ERR_ARG;
  uint64_t n_slots = 16;
  while (n_slots < (uint64_t)n_keys * 2) n_slots <<= 1;
  std::vector<NgramSlot> slots(n_slots, NgramSlot{~(uint64_t)0, -1, 0});
  for (int64_t r = 0; r < n_keys; ++r) {
    const uint64_t packed = ctx_len == 2 ? ((uint64_t)(uint32_t)keys[2 * r] << 32) |
                                               (uint32_t)keys[2 * r + 1]
                                         : (uint64_t)(uint32_t)keys[r];
    uint64_t h = mix64(packed) & (n_slots - 1);
    while (slots[h].key != ~(uint64_t)0) {
      if (slots[h].key == packed) return DART_ERR_ARG;   // duplicate context
      h = (h + 1) & (n_slots - 1);
    }
    slots[h].key = packed;
    slots[h].row = (int32_t)r;
  }
  const float miss = std::fmin(0.0f, (float)std::log(eps_d));
  const size_t cells = (size_t)std::max<int64_t>(n_keys, 1) * S;
  std::vector<int32_t> ids(cells, -1);
  std::vector<float> logp(cells, miss);
  // Rows are independent: scored (and validated) on a few host threads.  A used successor must
  // have a non-negative id, and the used ids of a row must be distinct: the pruning kernel lets
  // one thread per (successor, candidate) match write a score cell, so a duplicate would make
  // two threads write one cell with different values.
  std::vector<int> bad(8, 0);
  auto score_rows = [&](int64_t r0, int64_t r1, int *bad_flag) {
    int32_t seen[64];
    for (int64_t r = r0; r < r1; ++r) {
      int64_t total = 0;
      int used = 0;
      for (int j = 0; j < S; ++j) {
        const int32_t cnt = succ_counts[r * S + j];
        if (cnt < 0 || (cnt > 0 && succ_ids[r * S + j] < 0)) {
          *bad_flag = 1;
          return;
        }
        total += cnt;
        if (cnt > 0) seen[used++] = succ_ids[r * S + j];
      }
      std::sort(seen, seen + used);
      for (int j = 1; j < used; ++j)
        if (seen[j] == seen[j - 1]) {
          *bad_flag = 1;
          return;
        }
      for (int j = 0; j < S; ++j) {
        const int32_t cnt = succ_counts[r * S + j];
        if (cnt <= 0) continue;
        ids[r * S + j] = succ_ids[r * S + j];
        logp[r * S + j] = std::fmin(0.0f, (float)std::log(scale * (double)cnt / (double)total + eps_d));
      }
    }
  };
  {
    const int nthr = n_keys >= 4096 ? 8 : 1;
    std::vector<std::thread> pool;
    for (int i = 0; i < nthr; ++i)
      pool.emplace_back(score_rows, n_keys * i / nthr, n_keys * (i + 1) / nthr, &bad[i]);
    for (auto &th : pool) th.join();
    for (int i = 0; i < nthr; ++i)
      if (bad[i]) return DART_ERR_ARG;
  }
  hipError_t e = upload(slots.data(), n_slots * sizeof(NgramSlot), d_slots);
  if (e == hipSuccess) e = upload(ids.data(), cells * 4, d_ids);
  if (e == hipSuccess) e = upload(logp.data(), cells * 4, d_logp);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    for (void **q : {d_slots, d_ids, d_logp}) {
      if (*q) (void)hipFree(*q);
      *q = nullptr;
    }
    return from_hip(e);
  }
  *slot_mask = n_slots - 1;
  *miss_out = miss;
  return DART_OK;
}

dart_status dart_ngram_create(int n_gram, int64_t n_keys, int S, const int32_t *keys,
                              const int32_t *succ_ids, const int32_t *succ_counts, float eps,
                              dart_ngram **out) {
  if (!out) return DART_ERR_ARG;
  *out = nullptr;
  if ((n_gram != 2 && n_gram != 3) || n_keys < 0 || S < 1 || S > 64) return DART_ERR_ARG;
  if (n_keys > 0 && (!keys || !succ_ids || !succ_counts)) return DART_ERR_ARG;
  if (n_keys > ((int64_t)1 << 30)) return DART_ERR_ARG;
  dart_ngram *t = new (std::nothrow) dart_ngram();
  if (!t) return DART_ERR_OOM;
  std::memset(&t->dev, 0, sizeof t->dev);
  // s_ng = log(Pr + eps), Pr = count / sum of the row's counts (App. D)
  dart_status s = build_table(n_gram - 1, n_keys, S, keys, succ_ids, succ_counts, (double)eps, 1.0,
                              &t->slots, &t->succ_ids, &t->succ_logp, &t->dev.slot_mask,
                              &t->dev.logp_miss);
  if (s != DART_OK) {
    delete t;
    return s;
  }
  t->eps = eps;
  t->dev.n_gram = n_gram;
  t->dev.S = S;
  t->dev.slots = (const NgramSlot *)t->slots;
  t->dev.succ_ids = (const int32_t *)t->succ_ids;
  t->dev.succ_logp = (const float *)t->succ_logp;
  *out = t;
  return DART_OK;
}

dart_status dart_ngram_set_backoff(dart_ngram *t, int64_t n_keys, const int32_t *keys,
                                   const int32_t *succ_ids, const int32_t *succ_counts, float alpha) {
  if (!t) return DART_ERR_ARG;
  if (t->dev.n_gram != 3) return DART_ERR_ARG;            // the shorter context is one token
  if (n_keys < 0 || n_keys > ((int64_t)1 << 30)) return DART_ERR_ARG;
  if (n_keys > 0 && (!keys || !succ_ids || !succ_counts)) return DART_ERR_ARG;
  if (!(alpha > 0.0f) || !(alpha <= 1.0f)) return DART_ERR_ARG;
  void *slots = nullptr, *ids = nullptr, *logp = nullptr;
  uint64_t mask = 0;
  float miss = 0.f;
  dart_status s = build_table(1, n_keys, t->dev.S, keys, succ_ids, succ_counts, (double)t->eps,
                              (double)alpha, &slots, &ids, &logp, &mask, &miss);
  if (s != DART_OK) return s;
  // a table already attached is replaced; no kernel may be using it (see the header)
  for (void *q : {t->bo_slots, t->bo_succ_ids, t->bo_succ_logp})
    if (q) (void)hipFree(q);
  t->bo_slots = slots, t->bo_succ_ids = ids, t->bo_succ_logp = logp;
  t->dev.bo_slots = (const NgramSlot *)slots;
  t->dev.bo_slot_mask = mask;
  t->dev.bo_succ_ids = (const int32_t *)ids;
  t->dev.bo_succ_logp = (const float *)logp;
  return DART_OK;
}

void dart_ngram_destroy(dart_ngram *t) {
  if (!t) return;
  void *bufs[] = {t->slots, t->succ_ids, t->succ_logp, t->bo_slots, t->bo_succ_ids, t->bo_succ_logp};
  for (void *p : bufs)
    if (p) (void)hipFree(p);
  delete t;
}

dart_status dart_tree_prune(int batch, const int32_t *ids, const float *scores, int K,
                            const int32_t *ctx_tail, const dart_ngram *table,
                            const dart_prune_params *p, int32_t *tokens_out, int32_t *parents_out,
                            uint8_t *mask_out, int32_t *n_nodes_out, void *stream) {
  if (!ids || !scores || !ctx_tail || !table || !p || !tokens_out || !parents_out || !mask_out ||
      !n_nodes_out)
    return DART_ERR_ARG;
  if (batch < 1 || K < 1 || K > DART_MAX_K) return DART_ERR_ARG;
  if (p->k < 1 || p->k > DART_MAX_TOPK || p->beam_w < 1 || p->beam_w > DART_MAX_BEAM ||
      p->budget < 1 || p->budget > DART_MAX_BUDGET || p->beam_w * p->k > DART_MAX_LEVEL_NODES)
    return DART_ERR_ARG;
  // Alg. 1's "top-theta of T" is a tree only if scores never rise along a path: increments must
  // be <= 0, i.e. non-negative weights on scores that are <= 0 (as dart_topk and the table emit)
  if (!(p->w_ng >= 0.0f) || !(p->logit_decay > 0.0f) || !std::isfinite(p->w_ng) ||
      !std::isfinite(p->logit_decay) || !std::isfinite(p->level_pow))
    return DART_ERR_ARG;
  PruneLevelWeights lw;
  for (int L = 0; L < DART_MAX_K; ++L) {
    lw.w_logit[L] = (float)std::pow((double)p->logit_decay, (double)L);
    lw.w_level[L] = (float)std::pow((double)(L + 1), -(double)p->level_pow);
  }
  return from_hip(launch_prune(batch, ids, scores, K, ctx_tail, table->dev, *p, lw, tokens_out,
                               parents_out, mask_out, n_nodes_out, (hipStream_t)stream));
}

dart_status dart_tree_verify_greedy(int batch, const int32_t *tokens, const int32_t *parents,
                                    const int32_t *n_nodes, int budget, const int32_t *ctx_len,
                                    int32_t *position_ids, const int32_t *target_next,
                                    int path_cap, int32_t *accept_path, int32_t *n_accepted,
                                    int32_t *next_token, void *stream) {
  if (!tokens || !parents || !n_nodes) return DART_ERR_ARG;
  if (batch < 1 || budget < 1 || budget > DART_MAX_BUDGET || path_cap < 1) return DART_ERR_ARG;
  if (target_next && (!accept_path || !n_accepted || !next_token)) return DART_ERR_ARG;
  if (!target_next && !position_ids) return DART_ERR_ARG;      // nothing to do
  return from_hip(launch_tree_verify(batch, tokens, parents, n_nodes, target_next, ctx_len, budget,
                                     path_cap, position_ids, accept_path, n_accepted, next_token,
                                     (hipStream_t)stream));
}

#ifdef DART_TUNING
// Tuning builds only: set a kernel tunable by name (sweeps).  Returns 0 if the name is known.
int dart_debug_set(const char *name, int value) {
  if (!name) return -1;
  if (!strcmp(name, "gemv_wgs")) g_gemv_wgs = value;
  else if (!strcmp(name, "gemv_depth")) g_gemv_depth = value;
  else if (!strcmp(name, "gemv_xcd")) g_gemv_xcd = value;
  else if (!strcmp(name, "gemv_wgs_split")) g_gemv_wgs_split = value;
  else if (!strcmp(name, "gemv_nt")) g_gemv_nt = value;
  else if (!strcmp(name, "gemv_nt_min_mb")) g_gemv_nt_min_mb = value;
  else if (!strcmp(name, "gemv_split")) g_gemv_split = value;
  else if (!strcmp(name, "gemm_wgs")) g_gemm_wgs = value < 1 ? 1 : value;
  else if (!strcmp(name, "gemm_ord_map")) g_gemm_ord_map = value;
  else if (!strcmp(name, "attn_seg")) g_attn_seg = value < 0 ? 0 : (value > 64 ? 64 : value);
  else return -1;
  return 0;
}
#endif

// Diagnostic: run only the LM-head projection again on the final-normed rows the last forward
// call left in the workspace (used to time that kernel in isolation).
dart_status dart_debug_lm_head(dart_ctx *c, int rows, int multi_row, float *logits_out, void *stream) {
  if (!c || !logits_out || rows < 1 || rows > c->ws_rows) return DART_ERR_ARG;
  if (!multi_row && rows > DART_SKINNY_ROWS) return DART_ERR_ARG;
  if (multi_row && c->cfg.dtype != DART_BF16) return DART_ERR_ARG;
  if (multi_row == 2)      // contraction only: the operand tiles of the last LM-head call are reused
    return from_hip(launch_gemm_bf16(c->wlm, 0, (c->cfg.vocab + 15) / 16, nullptr, rows, c->xpack,
                                     logits_out, c->cfg.vocab, 0, 1, 0, (hipStream_t)stream));
  if (multi_row) {
    int chunks = 1;
    return from_hip(project(c, c->wlm, 0, c->cfg.vocab, c->yn, rows, logits_out, c->cfg.vocab, 0, 1, 1,
                            &chunks, (hipStream_t)stream));
  }
  return from_hip(lm_head(c, c->yn, rows, false, logits_out, (hipStream_t)stream));
}

// Diagnostic: only the candidate-selecting LM-head kernel of dart_draft_forward_topk, on the rows
// the last forward left behind; the per-workgroup lists stay in the workspace (no row merge).
dart_status dart_debug_lm_head_select(dart_ctx *c, int rows, int k, float *logits_out, void *stream) {
  if (!c || rows < 1 || rows > 8 || k < 1 || k > DART_MAX_TOPK || k > c->cfg.vocab) return DART_ERR_ARG;
  if (c->lm_select_wgs <= 0) return DART_ERR_STATE;
  const GemvTopk tk{c->topk_cand, c->topk_ms, k};
  int chunks = 1;
  return from_hip(launch_gemv_bf16(c->wlm, 0, (c->cfg.vocab + 15) / 16, c->yn, rows, logits_out,
                                   c->cfg.vocab, 0, 1, &chunks, (hipStream_t)stream, &tk));
}

// Diagnostic: which kernel, in which launch shape, dart_debug_lm_head (multi_row 0, 1 or 2) or
// dart_debug_lm_head_select (multi_row 3) runs.
int dart_debug_lm_head_key(dart_ctx *c, int rows, int multi_row, char *buf, int len) {
  if (!c || !buf || len < 1 || rows < 1 || c->cfg.dtype != DART_BF16) return -1;
  const int nstrips = (c->cfg.vocab + 15) / 16;
  if (multi_row == 3)
    return c->lm_select_wgs > 0 ? gemv_bf16_describe(c->wlm, nstrips, rows, 1, buf, len, true) : -1;
  if (multi_row) return gemm_bf16_describe(c->wlm, nstrips, rows, 1, 0, buf, len);
  return gemv_bf16_describe(c->wlm, nstrips, rows, gemv_bf16_chunks(c->cfg.d), buf, len);
}

// Diagnostic: copy a named fp32 workspace of the last forward to host memory (synchronises).
// Names: xn, resid, qkv, att_out, y, yn, hmid, u.  Returns the number of floats copied or -1.
int64_t dart_debug_read(dart_ctx *c, const char *name, float *host_out, int64_t max_count) {
  if (!c || !name || !host_out) return -1;
  const int R = DART_SKINNY_ROWS;
  const float *src = nullptr;
  int64_t count = 0;
  if (!strcmp(name, "xn")) src = c->xn, count = (int64_t)R * c->in_dim;
  else if (!strcmp(name, "resid")) src = c->resid, count = (int64_t)R * c->cfg.d;
  else if (!strcmp(name, "qkv")) src = c->qkv, count = (int64_t)R * c->qkv_dim;
  else if (!strcmp(name, "att_out")) src = c->att_out, count = (int64_t)R * c->q_dim;
  else if (!strcmp(name, "y")) src = c->y, count = (int64_t)R * c->cfg.d;
  else if (!strcmp(name, "yn")) src = c->yn, count = (int64_t)R * c->cfg.d;
  else if (!strcmp(name, "hmid")) src = c->hmid, count = (int64_t)R * c->cfg.ffn;
  else if (!strcmp(name, "u")) src = c->u, count = (int64_t)R * c->cfg.d;
  else return -1;
  if (count > max_count) count = max_count;
  if (hipDeviceSynchronize() != hipSuccess) return -1;
  if (hipMemcpy(host_out, src, count * 4, hipMemcpyDeviceToHost) != hipSuccess) return -1;
  return count;
}

}  // extern "C"
