// Host-side exercise of the C ABI's argument checks and error paths, built with
// -fsanitize=address,undefined on the host side (python -m paper_2601_19278_amd.build --sanitize)
// and run by tests/test_abi_sanitized.py.  Everything here returns before a kernel is launched;
// on a machine without a GPU the create calls with valid arguments fail inside the HIP runtime
// and must clean up after themselves, on a GPU machine they succeed and are destroyed again.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../include/dart.h"

static int failures = 0;
#define EXPECT(cond)                                              \
  do {                                                            \
    if (!(cond)) {                                                \
      std::printf("FAILED line %d: %s\n", __LINE__, #cond);       \
      ++failures;                                                 \
    }                                                             \
  } while (0)

int main() {
  for (int s = 0; s <= 6; ++s) EXPECT(std::strlen(dart_status_str((dart_status)s)) > 0);

  // ---- dart_create: configuration checks come before any device call
  dart_config cfg;
  std::memset(&cfg, 0, sizeof cfg);
  cfg.d = 64, cfg.n_q_heads = 2, cfg.n_kv_heads = 2, cfg.head_dim = 64, cfg.ffn = 64, cfg.vocab = 32;
  cfg.max_ctx = 8, cfg.max_K = 2, cfg.max_batch = 1, cfg.dtype = DART_F32, cfg.qk_norm = 0;
  cfg.rms_eps = 1e-6f, cfg.rope_base = 1e6f;
  std::vector<float> buf(64 * 128, 0.01f);
  dart_weights w;
  std::memset(&w, 0, sizeof w);
  const void *p = buf.data();
  w.w_in_norm = w.wq = w.wk = w.wv = w.wo = w.w_post_norm = w.w_gate = w.w_up = w.w_down = p;
  w.w_final_norm = w.w_lm = w.mask_emb = p;
  dart_ctx *ctx = nullptr;
  EXPECT(dart_create(nullptr, &w, &ctx) == DART_ERR_ARG);
  EXPECT(dart_create(&cfg, nullptr, &ctx) == DART_ERR_ARG);
  EXPECT(dart_create(&cfg, &w, nullptr) == DART_ERR_ARG);
  {
    dart_config bad = cfg;
    bad.head_dim = 32;
    EXPECT(dart_create(&bad, &w, &ctx) == DART_ERR_ARG && ctx == nullptr);
    bad = cfg, bad.n_q_heads = 3;
    EXPECT(dart_create(&bad, &w, &ctx) == DART_ERR_ARG);
    bad = cfg, bad.max_K = DART_MAX_K + 1;
    EXPECT(dart_create(&bad, &w, &ctx) == DART_ERR_ARG);
    bad = cfg, bad.vocab = 0;
    EXPECT(dart_create(&bad, &w, &ctx) == DART_ERR_ARG);
    bad = cfg, bad.d = 66;
    EXPECT(dart_create(&bad, &w, &ctx) == DART_ERR_ARG);
    bad = cfg, bad.dtype = 7;
    EXPECT(dart_create(&bad, &w, &ctx) == DART_ERR_ARG);
    bad = cfg, bad.max_ctx = 40000;
    EXPECT(dart_create(&bad, &w, &ctx) == DART_ERR_ARG);
    bad = cfg, bad.qk_norm = 1;                       // q_norm / k_norm missing
    EXPECT(dart_create(&bad, &w, &ctx) == DART_ERR_ARG);
    bad = cfg, bad.front_end = 1, bad.feat_dim = 192;  // front-end tensors missing
    EXPECT(dart_create(&bad, &w, &ctx) == DART_ERR_ARG);
    dart_weights w2 = w;
    w2.wq = nullptr;
    EXPECT(dart_create(&cfg, &w2, &ctx) == DART_ERR_ARG);
  }
  // valid arguments: succeeds on a GPU, fails cleanly (partly built context released) without one
  dart_status s = dart_create(&cfg, &w, &ctx);
  EXPECT(s == DART_OK || s == DART_ERR_HIP || s == DART_ERR_OOM);
  if (s == DART_OK) {
    EXPECT(dart_reset(ctx, 5) == DART_ERR_ARG);
    EXPECT(dart_reset(ctx, 0) == DART_OK);
    float dummy = 0.f;
    // argument errors of the forward and top-k calls: nothing is launched
    EXPECT(dart_draft_forward(ctx, 0, &dummy, 9, 0, 1, &dummy, nullptr) == DART_ERR_SHAPE);
    EXPECT(dart_draft_forward(ctx, 0, &dummy, 4, 0, 3, &dummy, nullptr) == DART_ERR_ARG);
    EXPECT(dart_draft_forward(ctx, 0, &dummy, 4, 2, 1, &dummy, nullptr) == DART_ERR_STATE);
    EXPECT(dart_draft_forward(ctx, 1, &dummy, 4, 0, 1, &dummy, nullptr) == DART_ERR_ARG);
    EXPECT(dart_draft_forward_features(ctx, 0, &dummy, nullptr, 4, 0, 1, &dummy, nullptr) == DART_ERR_ARG);
    int32_t i32 = 0;
    EXPECT(dart_topk(ctx, &dummy, 1, 64, 1, 1e-9f, &i32, &dummy, nullptr) == DART_ERR_SHAPE);
    EXPECT(dart_topk(ctx, &dummy, 1, 32, 33, 1e-9f, &i32, &dummy, nullptr) == DART_ERR_ARG);
    // the combined call: the forward's checks, then the top-k's; the logits buffer is optional
    EXPECT(dart_draft_forward_topk(ctx, 0, &dummy, 9, 0, 1, 1, 1e-9f, nullptr, &i32, &dummy, nullptr) == DART_ERR_SHAPE);
    EXPECT(dart_draft_forward_topk(ctx, 0, &dummy, 4, 2, 1, 1, 1e-9f, nullptr, &i32, &dummy, nullptr) == DART_ERR_STATE);
    EXPECT(dart_draft_forward_topk(ctx, 0, &dummy, 4, 0, 1, 0, 1e-9f, nullptr, &i32, &dummy, nullptr) == DART_ERR_ARG);
    EXPECT(dart_draft_forward_topk(ctx, 0, &dummy, 4, 0, 1, DART_MAX_TOPK + 1, 1e-9f, nullptr, &i32, &dummy, nullptr) == DART_ERR_ARG);
    EXPECT(dart_draft_forward_topk(ctx, 0, &dummy, 4, 0, 1, 1, 1e-9f, nullptr, nullptr, &dummy, nullptr) == DART_ERR_ARG);
    dart_destroy(ctx);
  } else {
    EXPECT(ctx == nullptr);
  }
  dart_destroy(nullptr);
  EXPECT(dart_reset(nullptr, 0) == DART_ERR_ARG);
  EXPECT(dart_draft_forward(nullptr, 0, nullptr, 1, 0, 1, nullptr, nullptr) == DART_ERR_ARG);
  EXPECT(dart_draft_forward_batched(nullptr, 1, nullptr, nullptr, nullptr, 1, nullptr, nullptr) == DART_ERR_ARG);
  EXPECT(dart_topk(nullptr, nullptr, 1, 1, 1, 1e-9f, nullptr, nullptr, nullptr) == DART_ERR_ARG);
  EXPECT(dart_draft_forward_topk(nullptr, 0, nullptr, 1, 0, 1, 1, 1e-9f, nullptr, nullptr, nullptr, nullptr) == DART_ERR_ARG);
  EXPECT(dart_draft_forward_features_topk(nullptr, 0, nullptr, nullptr, 1, 0, 1, 1, 1e-9f, nullptr, nullptr, nullptr,
                                          nullptr) == DART_ERR_ARG);
  EXPECT(dart_draft_forward_topk_batched(nullptr, 1, nullptr, nullptr, nullptr, 1, 1, 1e-9f, nullptr, nullptr, nullptr,
                                         nullptr) == DART_ERR_ARG);

  // ---- dart_topk_static: range checks come before the device is touched
  {
    float l = 0.f, sc = 0.f;
    int32_t id = 0;
    EXPECT(dart_topk_static(nullptr, 1, 8, 1, 1e-9f, &id, &sc, nullptr) == DART_ERR_ARG);
    EXPECT(dart_topk_static(&l, 0, 8, 1, 1e-9f, &id, &sc, nullptr) == DART_ERR_ARG);
    EXPECT(dart_topk_static(&l, 1, 8, 9, 1e-9f, &id, &sc, nullptr) == DART_ERR_ARG);
    EXPECT(dart_topk_static(&l, 1, 8, DART_MAX_TOPK + 1, 1e-9f, &id, &sc, nullptr) == DART_ERR_ARG);
    EXPECT(dart_topk_static(&l, DART_TOPK_STATIC_CELLS + 1, 8, 1, 1e-9f, &id, &sc, nullptr) == DART_ERR_SHAPE);
    EXPECT(dart_topk_static(&l, 2, 4096 * DART_TOPK_STATIC_CELLS, 1, 1e-9f, &id, &sc, nullptr) == DART_ERR_SHAPE);
  }

  // ---- dart_ngram_create: table validation runs on the host (threaded row pass included)
  {
    dart_ngram *t = nullptr;
    const int n = 5000, S = 4;                    // enough rows for the threaded pass
    std::vector<int32_t> keys(2 * n), ids(n * S), cnt(n * S, 1);
    for (int r = 0; r < n; ++r) {
      keys[2 * r] = r / 100, keys[2 * r + 1] = r % 100;
      for (int j = 0; j < S; ++j) ids[r * S + j] = (r * 7 + j * 13) % 1000 + j * 1000;
    }
    EXPECT(dart_ngram_create(4, n, S, keys.data(), ids.data(), cnt.data(), 1e-9f, &t) == DART_ERR_ARG);
    EXPECT(dart_ngram_create(3, n, 65, keys.data(), ids.data(), cnt.data(), 1e-9f, &t) == DART_ERR_ARG);
    EXPECT(dart_ngram_create(3, n, S, nullptr, ids.data(), cnt.data(), 1e-9f, &t) == DART_ERR_ARG);
    EXPECT(dart_ngram_create(3, n, S, keys.data(), ids.data(), cnt.data(), 1e-9f, nullptr) == DART_ERR_ARG);
    EXPECT(dart_ngram_create(3, -1, S, keys.data(), ids.data(), cnt.data(), 1e-9f, &t) == DART_ERR_ARG);
    auto expect_rejected = [&](int line) {
      dart_status st = dart_ngram_create(3, n, S, keys.data(), ids.data(), cnt.data(), 1e-9f, &t);
      if (st != DART_ERR_ARG || t != nullptr) {
        std::printf("FAILED line %d: table not rejected (status %d)\n", line, (int)st);
        ++failures;
      }
    };
    keys[2 * 4321] = -3;                           // negative context token
    expect_rejected(__LINE__);
    keys[2 * 4321] = 43;
    keys[2 * 4999] = keys[0], keys[2 * 4999 + 1] = keys[1];   // duplicate context
    expect_rejected(__LINE__);
    keys[2 * 4999] = 49, keys[2 * 4999 + 1] = 99;
    ids[4990 * S + 2] = -1;                        // used successor with a negative id
    expect_rejected(__LINE__);
    ids[4990 * S + 2] = ids[4990 * S + 1];         // successor repeated within its row
    expect_rejected(__LINE__);
    ids[4990 * S + 2] = 999999;
    cnt[17 * S] = -2;                              // negative count
    expect_rejected(__LINE__);
    cnt[17 * S] = 0;                               // an unused slot may hold any id
    ids[17 * S] = -1;
    s = dart_ngram_create(3, n, S, keys.data(), ids.data(), cnt.data(), 1e-9f, &t);
    EXPECT(s == DART_OK || s == DART_ERR_HIP || s == DART_ERR_OOM);
    if (s != DART_OK) EXPECT(t == nullptr);

    // ---- dart_tree_prune: parameter checks (the table pointer is only dereferenced after them)
    int32_t i32[64] = {0};
    float f32[64] = {0};
    uint8_t u8[64] = {0};
    const dart_ngram *tab = t ? t : reinterpret_cast<const dart_ngram *>(i32);   // never read on error
    dart_prune_params pp = {2, 2, 4, 0.5f, 0.9f, 0.7f};
    auto prune = [&](const dart_prune_params &q, int K, int batch) {
      return dart_tree_prune(batch, i32, f32, K, i32, tab, &q, i32, i32, u8, i32, nullptr);
    };
    EXPECT(dart_tree_prune(1, nullptr, f32, 2, i32, tab, &pp, i32, i32, u8, i32, nullptr) == DART_ERR_ARG);
    EXPECT(prune(pp, 0, 1) == DART_ERR_ARG);
    EXPECT(prune(pp, DART_MAX_K + 1, 1) == DART_ERR_ARG);
    EXPECT(prune(pp, 2, 0) == DART_ERR_ARG);
    dart_prune_params q = pp;
    q.k = 0;
    EXPECT(prune(q, 2, 1) == DART_ERR_ARG);
    q = pp, q.k = DART_MAX_TOPK + 1;
    EXPECT(prune(q, 2, 1) == DART_ERR_ARG);
    q = pp, q.beam_w = DART_MAX_BEAM + 1;
    EXPECT(prune(q, 2, 1) == DART_ERR_ARG);
    q = pp, q.budget = DART_MAX_BUDGET + 1;
    EXPECT(prune(q, 2, 1) == DART_ERR_ARG);
    q = pp, q.budget = 0;
    EXPECT(prune(q, 2, 1) == DART_ERR_ARG);
    q = pp, q.w_ng = -0.5f;
    EXPECT(prune(q, 2, 1) == DART_ERR_ARG);
    q = pp, q.logit_decay = 0.f;
    EXPECT(prune(q, 2, 1) == DART_ERR_ARG);
    q = pp, q.level_pow = NAN;
    EXPECT(prune(q, 2, 1) == DART_ERR_ARG);
    q = pp, q.w_ng = INFINITY;
    EXPECT(prune(q, 2, 1) == DART_ERR_ARG);
    EXPECT(dart_tree_verify_greedy(1, nullptr, i32, i32, 4, nullptr, i32, nullptr, 4, nullptr, nullptr,
                                   nullptr, nullptr) == DART_ERR_ARG);
    EXPECT(dart_tree_verify_greedy(1, i32, i32, i32, DART_MAX_BUDGET + 1, nullptr, i32, nullptr, 4, nullptr,
                                   nullptr, nullptr, nullptr) == DART_ERR_ARG);
    EXPECT(dart_tree_verify_greedy(1, i32, i32, i32, 4, nullptr, nullptr, i32, 4, nullptr, nullptr, nullptr,
                                   nullptr) == DART_ERR_ARG);
    dart_ngram_destroy(t);
    dart_ngram_destroy(nullptr);
  }
  if (failures == 0) std::printf("abi host check: ok\n");
  return failures == 0 ? 0 : 1;
}
