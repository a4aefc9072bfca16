"""GPU parity on seeded random shapes: the whole single-sequence step (forward with a random split
into cached and new rows, top-k through the combined call, pruning) against the oracle, stage by
stage, at shapes no other test fixes by hand (odd head counts per K/V head, ragged vocabulary and
context lengths, K from 1 to 12, fp32 and bf16, with and without q/k norm)."""
import numpy as np
import pytest

import dart_synth as ds
from oracle import draft_forward as odf, topk as otk, tree_prune as otp
from oracle.ngram import NgramModel
from util_gpu import hidden_to_device, logits_close, make_context

pytestmark = pytest.mark.gpu


def _random_config(rng):
    bf16 = bool(rng.integers(0, 4))                       # three bf16 cases for every fp32 one
    hd = int(rng.choice([64, 128]))
    n_kv = int(rng.choice([1, 2, 3, 4]))
    per = int(rng.choice([1, 2, 3, 4, 5, 8]))
    d = int(rng.choice([128, 256, 320, 512, 768])) if bf16 else int(rng.choice([64, 136, 256]))
    ffn = int(rng.choice([256, 352, 1024, 1536])) if bf16 else int(rng.choice([100, 256, 516]))
    K = int(rng.integers(1, 13))
    k = int(rng.integers(1, 13))
    vocab = int(rng.integers(max(k, 40), 30000))
    n_gram = int(rng.choice([2, 3]))
    return ds.scaled_config("C2" if bf16 else "C1", d=d, n_q_heads=n_kv * per, n_kv_heads=n_kv, head_dim=hd,
                            ffn=ffn, vocab=vocab, ctx=int(rng.integers(2, 330)), K=K, topk=k,
                            beam_w=int(rng.integers(1, 25)), budget=int(rng.integers(1, 80)), n_gram=n_gram,
                            n_keys=512, succ_per_key=int(rng.choice([4, 7, 16])), qk_norm=bool(rng.integers(0, 2)))


@pytest.mark.parametrize("seed", range(40))
def test_random_shape_step(seed):
    import torch
    import paper_2601_19278_amd as dart
    rng = np.random.default_rng(31000 + seed)
    cfg = _random_config(rng)
    tol = dict(atol=2e-2, rtol=1e-2) if cfg.dtype == "bf16" else dict(atol=2e-4, rtol=2e-4)
    ctx, W = make_context(cfg, 31100 + seed)
    counts = ds.make_ngram_counts(cfg, 31200 + seed)
    table = dart.NgramTable(cfg.n_gram, counts.keys, counts.succ_ids, counts.succ_counts, 1e-9)
    model = NgramModel(cfg.n_gram, counts.keys, counts.succ_ids, counts.succ_counts, 1e-9)
    hidden = ds.make_hidden(cfg, 31300 + seed)
    h = hidden_to_device(cfg, hidden)
    n, K, k = cfg.ctx, cfg.K, cfg.topk
    ref_logits = odf.draft_forward(cfg, W, hidden, K)
    # a first call over a random part of the prefix, then the rest with those rows cached
    part = int(rng.integers(1, n + 1))
    n_cached = 0
    if part < n:
        ctx.draft_forward(h, part, K)
        n_cached = int(rng.integers(0, part))             # at most part - 1 rows may be reused
    logits = torch.empty((K, cfg.vocab), dtype=torch.float32, device="cuda")
    ids, scores = ctx.draft_forward_topk(h, n, K, k, 1e-9, n_cached=n_cached, logits_out=logits)
    got = logits.cpu().numpy()
    ok, msg = logits_close(got, ref_logits, **tol)
    assert ok, f"{cfg}: {msg}"
    ref_ids, ref_scores = otk.topk_rows(got, k, 1e-9)
    np.testing.assert_array_equal(ids.cpu().numpy(), ref_ids)
    np.testing.assert_allclose(scores.cpu().numpy(), ref_scores, rtol=0, atol=1e-5)
    tail = counts.keys[int(rng.integers(0, len(counts.keys)))].astype(np.int32)
    gp = dart.PruneParams(k=k, beam_w=cfg.beam_w, budget=cfg.budget)
    tokens, parents, mask, n_nodes = table.tree_prune(ids, scores, torch.from_numpy(tail).cuda(), gp)
    ref = otp.tree_prune(ids.cpu().numpy(), scores.cpu().numpy(), tail, model,
                         otp.PruneParams(k=k, beam_w=cfg.beam_w, budget=cfg.budget))
    assert int(n_nodes.cpu()) == ref.n_nodes
    np.testing.assert_array_equal(tokens.cpu().numpy()[0] if tokens.dim() == 2 else tokens.cpu().numpy(), ref.tokens)
    np.testing.assert_array_equal(parents.cpu().numpy().reshape(-1), ref.parents)
    np.testing.assert_array_equal(mask.cpu().numpy().reshape(ref.mask.shape), ref.mask)
    ctx.close()
    table.close()


@pytest.mark.parametrize("seed", range(12))
def test_random_shape_batched_step(seed):
    """The batched calls (multi-row kernels) on random bf16 shapes and batch sizes: ragged lengths, a
    random cached part per sequence, the combined forward + top-k call, pruning of the whole batch."""
    import torch
    import paper_2601_19278_amd as dart
    rng = np.random.default_rng(32000 + seed)
    cfg = _random_config(rng)
    while cfg.dtype != "bf16":
        cfg = _random_config(rng)
    B = int(rng.integers(1, 21))
    from dataclasses import replace
    cfg = replace(cfg, batch=B, K=min(cfg.K, 8))
    K, k = cfg.K, cfg.topk
    ctx, W = make_context(cfg, 32100 + seed)
    counts = ds.make_ngram_counts(cfg, 32200 + seed)
    table = dart.NgramTable(cfg.n_gram, counts.keys, counts.succ_ids, counts.succ_counts, 1e-9)
    model = NgramModel(cfg.n_gram, counts.keys, counts.succ_ids, counts.succ_counts, 1e-9)
    lens = [int(v) for v in rng.integers(1, cfg.ctx + 1, size=B)]
    hiddens = [ds.make_hidden(cfg, 32300 + 50 * seed + b, n=lens[b]) for b in range(B)]
    devs = [hidden_to_device(cfg, h) for h in hiddens]
    part = [int(rng.integers(1, n + 1)) for n in lens]
    ctx.draft_forward_batched(devs, part, [0] * B, K)
    cached = [int(rng.integers(0, p)) if p < n else int(rng.integers(0, n)) for p, n in zip(part, lens)]
    logits = torch.empty((B, K, cfg.vocab), dtype=torch.float32, device="cuda")
    ids, scores = ctx.draft_forward_topk_batched(devs, lens, cached, K, k, 1e-9, logits_out=logits)
    got = logits.cpu().numpy()
    for b in range(B):
        ok, msg = logits_close(got[b], odf.draft_forward(cfg, W, hiddens[b], K), atol=2e-2, rtol=1e-2)
        assert ok, f"{cfg} sequence {b} (n={lens[b]}, cached={cached[b]}): {msg}"
    ref_ids, ref_scores = otk.topk_rows(got.reshape(B * K, cfg.vocab), k, 1e-9)
    np.testing.assert_array_equal(ids.cpu().numpy().reshape(B * K, k), ref_ids)
    np.testing.assert_allclose(scores.cpu().numpy().reshape(B * K, k), ref_scores, rtol=0, atol=1e-5)
    tails = np.ascontiguousarray(counts.keys[rng.integers(0, len(counts.keys), size=B)].astype(np.int32))
    gp = dart.PruneParams(k=k, beam_w=cfg.beam_w, budget=cfg.budget)
    tokens, parents, mask, n_nodes = [t.cpu().numpy() for t in
                                      table.tree_prune(ids, scores, torch.from_numpy(tails).cuda(), gp)]
    ids_h, scores_h = ids.cpu().numpy(), scores.cpu().numpy()
    for b in range(B):
        ref = otp.tree_prune(ids_h[b], scores_h[b], tails[b], model,
                             otp.PruneParams(k=k, beam_w=cfg.beam_w, budget=cfg.budget))
        assert int(n_nodes[b]) == ref.n_nodes, b
        np.testing.assert_array_equal(tokens[b], ref.tokens)
        np.testing.assert_array_equal(parents[b], ref.parents)
        np.testing.assert_array_equal(mask[b], ref.mask)
    ctx.close()
    table.close()
