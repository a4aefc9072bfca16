"""GPU parity: dart_draft_forward_topk -- the LM head that selects its workgroups' candidates itself
(Alg. 1 "Top-k_i tokens from l_i", App. D "s_logit") -- against dart_draft_forward + dart_topk and
against the oracle's full sort on the logits the same call wrote."""
import numpy as np
import pytest

import dart_synth as ds
from oracle import topk as otk
from util_gpu import hidden_to_device, make_context

pytestmark = pytest.mark.gpu

SHAPES = {
    # LM-head strips not a whole number per workgroup, vocabulary not a multiple of 16
    "ragged_vocab": ds.scaled_config("C2", d=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=512,
                                     vocab=40007, ctx=70, K=5),
    "mid": ds.scaled_config("C2", d=512, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn=1536,
                            vocab=151936, ctx=130, K=8),
    # fewer strips than workgroups: most workgroups hold one strip, some none
    "tiny_vocab": ds.scaled_config("C2", d=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=512,
                                   vocab=1000, ctx=33, K=3),
}


def _check(cfg, seed, ks=(1, 10, 64), K=None):
    import torch
    K = cfg.K if K is None else K
    ctx, W = make_context(cfg, seed)
    hidden = ds.make_hidden(cfg, seed + 1)
    h = hidden_to_device(cfg, hidden)
    n = cfg.ctx
    plain = ctx.draft_forward(h, n, K).cpu().numpy()
    for k in ks:
        k = min(k, cfg.vocab)
        logits = torch.full((K, cfg.vocab), 7.0, dtype=torch.float32, device="cuda")
        ctx.reset()
        ids, scores = ctx.draft_forward_topk(h, n, K, k, 1e-9, logits_out=logits)
        got = logits.cpu().numpy()
        np.testing.assert_array_equal(got, plain)                  # the same logits, bit for bit
        ref_ids, ref_scores = otk.topk_rows(got, k, 1e-9)
        np.testing.assert_array_equal(ids.cpu().numpy(), ref_ids)  # ids and order: bit-exact
        np.testing.assert_allclose(scores.cpu().numpy(), ref_scores, rtol=0, atol=1e-5)
        two_ids, two_scores = ctx.topk(logits, k, 1e-9)            # the two-call route
        assert torch.equal(ids, two_ids)
        np.testing.assert_allclose(scores.cpu().numpy(), two_scores.cpu().numpy(), rtol=0, atol=2e-6)
        # warm call without a logits buffer: candidates only, identical
        ids2, scores2 = ctx.draft_forward_topk(h, n, K, k, 1e-9, n_cached=n - 1)
        assert torch.equal(ids2, ids) and torch.equal(scores2, scores)
    ctx.close()


@pytest.mark.parametrize("name", sorted(SHAPES))
def test_small_shapes(name):
    _check(SHAPES[name], 8100)


def test_more_than_eight_rows_and_fp32_take_the_two_step_route():
    _check(ds.scaled_config("C2", d=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=512, vocab=5000,
                            ctx=40, K=12), 8200, ks=(7,))
    _check(ds.get_config("C1"), 8300, ks=(4,))


def test_planted_ties_across_workgroups():
    """Equal logits in different workgroups' strips and at the top-k boundary: a weight matrix
    with repeated LM-head rows gives exactly equal logits; ids must come out in ascending order."""
    import torch
    import paper_2601_19278_amd as dart
    cfg = SHAPES["mid"]
    W = ds.make_weights(cfg, 8400)
    lm = W["w_lm"].copy()
    src = lm[12345].copy()
    for v in (0, 17, 5000, 70001, 151935, 99999, 64, 65, 151920):    # copies spread over the vocabulary
        lm[v] = src
    W["w_lm"] = lm
    ctx = dart.DraftContext(cfg, W)
    hidden = ds.make_hidden(cfg, 8401)
    h = hidden_to_device(cfg, hidden)
    logits = torch.empty((cfg.K, cfg.vocab), dtype=torch.float32, device="cuda")
    for k in (3, 10, 12):
        ctx.reset()
        ids, scores = ctx.draft_forward_topk(h, cfg.ctx, cfg.K, k, 1e-9, logits_out=logits)
        got = logits.cpu().numpy()
        assert (got[:, [0, 17, 5000, 70001]] == got[:, [12345]]).all()
        ref_ids, ref_scores = otk.topk_rows(got, k, 1e-9)
        np.testing.assert_array_equal(ids.cpu().numpy(), ref_ids)
        np.testing.assert_allclose(scores.cpu().numpy(), ref_scores, rtol=0, atol=1e-5)
    ctx.close()


def test_c4_headline_full_size_and_determinism():
    import torch
    cfg = ds.get_config("C4")
    ctx, W = make_context(cfg, 4000)
    hidden = ds.make_hidden(cfg, 4001)
    h = hidden_to_device(cfg, hidden)
    n, K, k = cfg.ctx, cfg.K, cfg.topk
    logits = torch.empty((K, cfg.vocab), dtype=torch.float32, device="cuda")
    ids, scores = ctx.draft_forward_topk(h, n, K, k, 1e-9, logits_out=logits)
    got = logits.cpu().numpy()
    ref_ids, ref_scores = otk.topk_rows(got, k, 1e-9)
    np.testing.assert_array_equal(ids.cpu().numpy(), ref_ids)
    np.testing.assert_allclose(scores.cpu().numpy(), ref_scores, rtol=0, atol=1e-5)
    np.testing.assert_array_equal(got, ctx.draft_forward(h, n, K, n_cached=n - 4).cpu().numpy())
    for _ in range(10):                                           # repeated runs are bit-identical
        ids2, scores2 = ctx.draft_forward_topk(h, n, K, k, 1e-9, n_cached=n - 4)
        assert torch.equal(ids2, ids) and torch.equal(scores2, scores)
    ctx.close()


def test_error_statuses():
    import torch
    import paper_2601_19278_amd as dart
    cfg = SHAPES["tiny_vocab"]
    ctx, _ = make_context(cfg, 8500)
    h = hidden_to_device(cfg, ds.make_hidden(cfg, 8501))
    for kwargs, status in ((dict(k=0), 1), (dict(k=65), 1), (dict(K=cfg.K + 1), 1), (dict(n_cached=cfg.ctx), 5)):
        args = dict(ctx_len=cfg.ctx, K=cfg.K, k=3)
        args.update(kwargs)
        with pytest.raises(dart.DartError) as ei:
            ctx.draft_forward_topk(h, args.pop("ctx_len"), args.pop("K"), args.pop("k"), 1e-9, **args)
        assert ei.value.status == status, kwargs
    ctx.close()
