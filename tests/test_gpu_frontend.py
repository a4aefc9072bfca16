"""GPU parity: dart_draft_forward_features (FC + shifted embeddings front end, 2d-wide attention
input) against the oracle."""
import numpy as np
import pytest

import dart_synth as ds
from oracle import draft_forward as odf
from util_gpu import hidden_to_device, logits_close

pytestmark = pytest.mark.gpu

F32_TOL = dict(atol=2e-4, rtol=2e-4)
BF16_TOL = dict(atol=2e-2, rtol=1e-2)

CASES = {
    # fp32, bigger feature width than 3d is allowed; K/V heads = query heads
    "f32": (ds.scaled_config("C1", d=256, n_q_heads=4, n_kv_heads=4, head_dim=64, ffn=512, vocab=3000,
                             ctx=70, K=4), 3 * 256),
    # bf16, ragged sizes: vocab not a multiple of 16, context not a multiple of 32
    "bf16_small": (ds.scaled_config("C2", d=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=512,
                                    vocab=1000, ctx=70, K=5), 3 * 256),
    # bf16, hd 128, FC and QKV inputs long enough for several k-chunks
    "bf16_mid": (ds.scaled_config("C2", d=1024, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn=2048,
                                  vocab=8192, ctx=300, K=8), 3 * 1024),
}


def _ctx(cfg, W, feat_dim):
    import paper_2601_19278_amd as dart
    return dart.DraftContext(cfg, W, feat_dim=feat_dim)


@pytest.mark.parametrize("name", sorted(CASES))
def test_front_end_matches_oracle_cold_and_warm(name):
    import torch
    cfg, feat_dim = CASES[name]
    W = ds.make_frontend_weights(cfg, 6000, feat_dim=feat_dim)
    feats, toks = ds.make_features(cfg, 6001, feat_dim=feat_dim)
    ref = odf.draft_forward_features(cfg, W, feats, toks, cfg.K)
    ctx = _ctx(cfg, W, feat_dim)
    f_dev, t_dev = hidden_to_device(cfg, feats), torch.from_numpy(toks).cuda()
    tol = BF16_TOL if cfg.dtype == "bf16" else F32_TOL
    n = cfg.ctx
    first = None
    for n_cached in (0, n - 1, n - 4, 9, 0):
        if n_cached == 0:
            ctx.reset()
        out = ctx.draft_forward_features(f_dev, t_dev, n, cfg.K, n_cached=n_cached).cpu().numpy()
        ok, msg = logits_close(out, ref, **tol)
        assert ok, f"{name} n_cached={n_cached}: {msg}"
        if first is None:
            first = out
        else:
            np.testing.assert_array_equal(out, first)       # cold and warm agree bit for bit
    ctx.close()


def test_front_end_growing_prefix_and_entry_point_guards():
    import torch
    import paper_2601_19278_amd as dart
    cfg, feat_dim = CASES["bf16_small"]
    W = ds.make_frontend_weights(cfg, 6100, feat_dim=feat_dim)
    feats, toks = ds.make_features(cfg, 6101, feat_dim=feat_dim)
    ctx = _ctx(cfg, W, feat_dim)
    f_dev, t_dev = hidden_to_device(cfg, feats), torch.from_numpy(toks).cuda()
    cached = 0
    for n in (12, 13, 17, 40, 70):
        # the token after the last position is the freshly sampled one: it changes from step to step
        toks_n = toks[:n].copy()
        toks_n[-1] = (toks[n - 1] + 7) % cfg.vocab
        t_n = torch.from_numpy(toks_n).cuda()
        out = ctx.draft_forward_features(f_dev, t_n, n, cfg.K, n_cached=cached).cpu().numpy()
        ref = odf.draft_forward_features(cfg, W, feats[:n], toks_n, cfg.K)
        ok, msg = logits_close(out, ref, **BF16_TOL)
        assert ok, (n, msg)
        cached = n - 1        # the last row's embedding was provisional: its K/V are recomputed
    with pytest.raises(dart.DartError) as ei:
        ctx.draft_forward(f_dev, 10, 2)                      # fused-input call on a front-end context
    assert ei.value.status == 5
    with pytest.raises(dart.DartError) as ei:
        ctx.draft_forward_topk(f_dev, 10, 2, 3)
    assert ei.value.status == 5
    ctx.close()
    plain = dart.DraftContext(cfg, ds.make_weights(cfg, 6100))
    with pytest.raises(dart.DartError) as ei:
        plain.draft_forward_features(f_dev, t_dev, 10, 2)
    assert ei.value.status == 5
    with pytest.raises(dart.DartError) as ei:
        plain.draft_forward_features_topk(f_dev, t_dev, 10, 2, 3)
    assert ei.value.status == 5
    plain.close()


def test_front_end_full_size_1p7b_shapes():
    """Preset C2's shapes with the front end: feat_dim = 3 d = 6144, vocabulary 151936."""
    import torch
    cfg = ds.get_config("C2")
    feat_dim = 3 * cfg.d
    W = ds.make_frontend_weights(cfg, 6200, feat_dim=feat_dim)
    feats, toks = ds.make_features(cfg, 6201, feat_dim=feat_dim)
    ref = odf.draft_forward_features(cfg, W, feats, toks, cfg.K)
    ctx = _ctx(cfg, W, feat_dim)
    f_dev, t_dev = hidden_to_device(cfg, feats), torch.from_numpy(toks).cuda()
    cold = ctx.draft_forward_features(f_dev, t_dev, cfg.ctx, cfg.K).cpu().numpy()
    ok, msg = logits_close(cold, ref, **BF16_TOL)
    assert ok, msg
    warm = ctx.draft_forward_features(f_dev, t_dev, cfg.ctx, cfg.K, n_cached=cfg.ctx - 4).cpu().numpy()
    np.testing.assert_array_equal(warm, cold)
    # forward + top-k as one call: the same logits, candidates bit-exact against the full sort
    from oracle import topk as otk
    lg = torch.empty((cfg.K, cfg.vocab), dtype=torch.float32, device="cuda")
    ids, scores = ctx.draft_forward_features_topk(f_dev, t_dev, cfg.ctx, cfg.K, cfg.topk, 1e-9,
                                                  n_cached=cfg.ctx - 4, logits_out=lg)
    np.testing.assert_array_equal(lg.cpu().numpy(), cold)
    ref_ids, ref_scores = otk.topk_rows(cold, cfg.topk, 1e-9)
    np.testing.assert_array_equal(ids.cpu().numpy(), ref_ids)
    np.testing.assert_allclose(scores.cpu().numpy(), ref_scores, rtol=0, atol=1e-5)
    ids2, scores2 = ctx.draft_forward_features_topk(f_dev, t_dev, cfg.ctx, cfg.K, cfg.topk, 1e-9,
                                                    n_cached=cfg.ctx - 1)
    assert torch.equal(ids2, ids) and torch.equal(scores2, scores)
    ctx.close()


@pytest.mark.parametrize("name", ["bf16_small", "bf16_mid"])
def test_front_end_batched_matches_oracle_cold_and_warm(name):
    """dart_draft_forward_features_batched: ragged sequences share every launch (FC and the other
    projections on the multi-row kernel); each sequence against the oracle, and a warm call
    reproduces the cold one bit for bit."""
    import torch
    import paper_2601_19278_amd as dart
    cfg, feat_dim = CASES[name]
    lens = [cfg.ctx, 17, cfg.ctx // 2 + 3, 64, 1]
    W = ds.make_frontend_weights(cfg, 6300, feat_dim=feat_dim)
    seqs = [ds.make_features(cfg, 6301 + b, n=n, feat_dim=feat_dim) for b, n in enumerate(lens)]
    refs = [odf.draft_forward_features(cfg, W, f, t, cfg.K) for f, t in seqs]
    ctx = dart.DraftContext(cfg, W, max_batch=len(lens), feat_dim=feat_dim)
    f_dev = [hidden_to_device(cfg, f) for f, _ in seqs]
    t_dev = [torch.from_numpy(t).cuda() for _, t in seqs]
    cold = ctx.draft_forward_features_batched(f_dev, t_dev, lens, [0] * len(lens), cfg.K).cpu().numpy()
    for b in range(len(lens)):
        ok, msg = logits_close(cold[b], refs[b], **BF16_TOL)
        assert ok, f"{name} sequence {b} (n={lens[b]}): {msg}"
    for cached in ([n - 1 for n in lens], [max(0, n - 5) for n in lens], [0, 16, 3, 63, 0]):
        warm = ctx.draft_forward_features_batched(f_dev, t_dev, lens, cached, cfg.K).cpu().numpy()
        np.testing.assert_array_equal(warm, cold)
    # the fused-input batched call is refused on a front-end context
    with pytest.raises(dart.DartError) as ei:
        ctx.draft_forward_batched(f_dev, lens, [0] * len(lens), cfg.K)
    assert ei.value.status == 5
    ctx.close()
