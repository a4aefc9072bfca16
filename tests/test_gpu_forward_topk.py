"""GPU parity: dart_draft_forward_topk -- the LM head that selects its workgroups' candidates itself
(Alg. 1 "Top-k_i tokens from l_i", App. D "s_logit") -- and dart_draft_forward_topk_batched, against
the separate forward and top-k calls and against the oracle's full sort on the logits the same call
wrote."""
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


# ---- batched: dart_draft_forward_topk_batched (multi-row forward, then the top-k kernels) ----

BATCHED = [
    # 128 rows: 8 row tiles, vocabulary ragged in its last strip
    (16, 8, dict(d=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=512, vocab=40007, ctx=60)),
    # 48 rows (4 row tiles, last tile absent rows), one or two strips per wavefront
    (6, 8, dict(d=512, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn=1536, vocab=8200, ctx=90)),
    # 6 rows of 32 (2 row tiles), wide vocabulary: 37-38 strips per workgroup, five per wavefront
    (2, 3, dict(d=256, n_q_heads=2, n_kv_heads=1, head_dim=128, ffn=512, vocab=151936, ctx=40)),
    # fewer strips than workgroups x wavefronts: most wavefronts hold no strip
    (16, 8, dict(d=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=512, vocab=1000, ctx=33)),
    # two groups of sequences (20 > 16): the second group's candidates land behind the first's
    (20, 2, dict(d=256, n_q_heads=4, n_kv_heads=4, head_dim=64, ffn=512, vocab=2048, ctx=40)),
    # 16 x 12 = 192 rows: more than one row block, the two-step route
    (16, 12, dict(d=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=512, vocab=3000, ctx=40)),
]


def _batched_inputs(cfg, batch, seed):
    rng = np.random.default_rng(seed)
    lens = [int(v) for v in rng.integers(5, cfg.ctx + 1, size=batch)]
    lens[0] = cfg.ctx
    hiddens = [ds.make_hidden(cfg, seed + 1 + b, n=lens[b]) for b in range(batch)]
    return lens, [hidden_to_device(cfg, h) for h in hiddens]


def _check_batched(ctx, cfg, devs, lens, batch, K, ks):
    import torch
    plain = ctx.draft_forward_batched(devs, lens, [0] * batch, K).cpu().numpy()
    for k in ks:
        k = min(k, cfg.vocab)
        logits = torch.full((batch, K, cfg.vocab), 7.0, dtype=torch.float32, device="cuda")
        ids, scores = ctx.draft_forward_topk_batched(devs, lens, [0] * batch, K, k, 1e-9, logits_out=logits)
        got = logits.cpu().numpy()
        np.testing.assert_array_equal(got, plain)                    # the same logits, bit for bit
        ref_ids, ref_scores = otk.topk_rows(got.reshape(batch * K, cfg.vocab), k, 1e-9)
        np.testing.assert_array_equal(ids.cpu().numpy().reshape(batch * K, k), ref_ids)
        np.testing.assert_allclose(scores.cpu().numpy().reshape(batch * K, k), ref_scores, rtol=0, atol=1e-5)
        # warm call without a logits buffer: candidates only, identical
        warm = [n - 1 for n in lens]
        ids2, scores2 = ctx.draft_forward_topk_batched(devs, lens, warm, K, k, 1e-9)
        assert torch.equal(ids2, ids) and torch.equal(scores2, scores)


@pytest.mark.parametrize("batch,K,over", BATCHED)
def test_batched_small_shapes(batch, K, over):
    cfg = ds.scaled_config("C2", K=K, batch=batch, **over)
    ctx, W = make_context(cfg, 8600)
    lens, devs = _batched_inputs(cfg, batch, 8601)
    _check_batched(ctx, cfg, devs, lens, batch, K, ks=(1, 10, 16, 64))
    ctx.close()


def test_batched_many_equal_logits():
    """Runs of identical LM-head rows give that many equal logits in every one of the 128 rows: the
    selection's candidate buffers overflow and the sequential extraction takes over; ids must still
    come out in ascending order among equals."""
    import paper_2601_19278_amd as dart
    batch, K = 16, 8
    cfg = ds.scaled_config("C2", K=K, batch=batch, d=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=512,
                           vocab=40007, ctx=40)
    W = ds.make_weights(cfg, 8700)
    lm = W["w_lm"].copy()
    lm[3000:3200] = lm[17]            # 200 equal logits in a row, inside one or two ranges
    lm[39990:40007] = lm[17]          # and in the ragged last strip
    lm[20000:20040] = lm[5]           # a shorter run that fits a list
    W["w_lm"] = lm
    ctx = dart.DraftContext(cfg, W)
    lens, devs = _batched_inputs(cfg, batch, 8701)
    _check_batched(ctx, cfg, devs, lens, batch, K, ks=(10, 30))
    ctx.close()


def test_c5_batched_headline_full_size_and_determinism():
    import torch
    from dart_synth.tensors import make_ragged_lengths
    cfg = ds.get_config("C5")
    B, K, k = cfg.batch, cfg.K, cfg.topk
    ctx, W = make_context(cfg, 5000)
    lens = [min(n, 600) for n in make_ragged_lengths(cfg, 5001).tolist()]    # short prefixes: the LM head is the subject
    devs = [hidden_to_device(cfg, ds.make_hidden(cfg, 5002 + b, n=lens[b])) for b in range(B)]
    logits = torch.empty((B, K, cfg.vocab), dtype=torch.float32, device="cuda")
    ids, scores = ctx.draft_forward_topk_batched(devs, lens, [0] * B, K, k, 1e-9, logits_out=logits)
    got = logits.cpu().numpy().reshape(B * K, cfg.vocab)
    ref_ids, ref_scores = otk.topk_rows(got, k, 1e-9)
    np.testing.assert_array_equal(ids.cpu().numpy().reshape(B * K, k), ref_ids)
    np.testing.assert_allclose(scores.cpu().numpy().reshape(B * K, k), ref_scores, rtol=0, atol=1e-5)
    assert torch.equal(logits, ctx.draft_forward_batched(devs, lens, [n - 1 for n in lens], K))
    for _ in range(10):                                           # repeated runs are bit-identical
        ids2, scores2 = ctx.draft_forward_topk_batched(devs, lens, [n - 1 for n in lens], K, k, 1e-9)
        assert torch.equal(ids2, ids) and torch.equal(scores2, scores)
    ctx.close()
