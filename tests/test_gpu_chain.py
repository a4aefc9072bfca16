"""GPU parity of the whole draft step chained on the device: dart_draft_forward -> dart_topk ->
dart_tree_prune, each stage checked against the oracle on the inputs that stage actually saw."""
import numpy as np
import pytest

import dart_synth as ds
from oracle import draft_forward as odf, topk as otk, tree_prune as otp
from oracle.ngram import NgramModel
from util_gpu import hidden_to_device, logits_close, make_context

pytestmark = pytest.mark.gpu


def _chain(cfg, ctx, table, hidden, tail, n_cached=0):
    import torch
    import paper_2601_19278_amd as dart
    h = hidden_to_device(cfg, hidden)
    logits = ctx.draft_forward(h, hidden.shape[0], cfg.K, n_cached=n_cached)
    ids, scores = ctx.topk(logits, cfg.topk, 1e-9)
    params = dart.PruneParams(k=cfg.topk, beam_w=cfg.beam_w, budget=cfg.budget)
    tree = table.tree_prune(ids, scores, torch.from_numpy(tail).cuda(), params)
    torch.cuda.synchronize()
    return [t.cpu().numpy() for t in (logits, ids, scores, *tree)]


def _check_stages(cfg, W, model, hidden, tail, got, tol):
    logits, ids, scores, tokens, parents, mask, n_nodes = got
    ref_logits = odf.draft_forward(cfg, W, hidden, cfg.K)
    ok, msg = logits_close(logits, ref_logits, **tol)
    assert ok, msg
    # top-k on the very buffer the kernel read: ids and order bit-exact
    ref_ids, ref_scores = otk.topk_rows(logits, cfg.topk, 1e-9)
    np.testing.assert_array_equal(ids, ref_ids)
    np.testing.assert_allclose(scores, ref_scores, rtol=0, atol=1e-5)
    # chained ids against the oracle's own logits wherever the oracle's rank gaps exceed twice
    # the logit tolerance (closer calls may legitimately swap)
    oid, _ = otk.topk_rows(ref_logits, cfg.topk + 1, 1e-9)
    skipped = 0
    for r in range(cfg.K):
        vals = ref_logits[r, oid[r]]
        gaps = -np.diff(vals)
        bound = 2 * (tol["atol"] + tol["rtol"] * np.abs(vals[:-1]))
        if (gaps > bound).all():
            np.testing.assert_array_equal(ids[r], oid[r, : cfg.topk])
        else:
            skipped += 1
    # pruning on the candidates the kernel was given: tree bit-exact
    ref = otp.tree_prune(ids, scores, tail, model,
                         otp.PruneParams(k=cfg.topk, beam_w=cfg.beam_w, budget=cfg.budget))
    assert int(n_nodes) == ref.n_nodes
    np.testing.assert_array_equal(tokens, ref.tokens)
    np.testing.assert_array_equal(parents, ref.parents)
    np.testing.assert_array_equal(mask, ref.mask)
    return skipped


def test_c1_chain_many_seeds_and_determinism():
    import paper_2601_19278_amd as dart
    cfg = ds.get_config("C1")
    ctx, W = make_context(cfg, 9000)
    counts = ds.make_ngram_counts(cfg, 9001)
    table = dart.NgramTable(cfg.n_gram, counts.keys, counts.succ_ids, counts.succ_counts, 1e-9)
    model = NgramModel(cfg.n_gram, counts.keys, counts.succ_ids, counts.succ_counts, 1e-9)
    tol = dict(atol=2e-4, rtol=2e-4)
    rng = np.random.default_rng(9002)
    skipped = 0
    for seed in range(100):
        hidden = ds.make_hidden(cfg, 9100 + seed)
        tail = rng.integers(0, cfg.vocab, size=cfg.n_gram - 1).astype(np.int32)
        ctx.reset()
        got = _chain(cfg, ctx, table, hidden, tail)
        skipped += _check_stages(cfg, W, model, hidden, tail, got, tol)
    assert skipped < 100 * cfg.K // 2            # most rows have clear gaps at fp32 accuracy
    first = _chain(cfg, ctx, table, hidden, tail, n_cached=cfg.ctx - 1)
    for _ in range(50):                           # repeated runs are bit-identical
        again = _chain(cfg, ctx, table, hidden, tail, n_cached=cfg.ctx - 1)
        for a, b in zip(first, again):
            np.testing.assert_array_equal(a, b)
    ctx.close()
    table.close()


@pytest.mark.parametrize("name", ["C2", "C3", "C4"])
def test_full_size_chain_with_preset_table(name):
    """Whole step at a bf16 preset with its 2^20-context trigram table (random-init logits give
    near-uniform candidates, so most lookups miss; hits are covered by the planted prune cases)."""
    import paper_2601_19278_amd as dart
    cfg = ds.get_config(name)
    seed = 9500 + int(name[1:])
    ctx, W = make_context(cfg, seed)
    counts = ds.make_ngram_counts(cfg, seed + 1)
    table = dart.NgramTable(cfg.n_gram, counts.keys, counts.succ_ids, counts.succ_counts, 1e-9)
    model = NgramModel(cfg.n_gram, counts.keys, counts.succ_ids, counts.succ_counts, 1e-9)
    hidden = ds.make_hidden(cfg, seed + 2)
    tail = counts.keys[123].astype(np.int32)       # a stored context: level 0 looks up a real row
    got = _chain(cfg, ctx, table, hidden, tail)
    _check_stages(cfg, W, model, hidden, tail, got, dict(atol=2e-2, rtol=1e-2))
    # the combined forward + top-k call (warm) gives the same candidates as the two calls
    import torch
    h = hidden_to_device(cfg, hidden)
    ids_f, scores_f = ctx.draft_forward_topk(h, hidden.shape[0], cfg.K, cfg.topk, 1e-9, n_cached=hidden.shape[0] - 1)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(ids_f.cpu().numpy(), got[1])
    np.testing.assert_allclose(scores_f.cpu().numpy(), got[2], rtol=0, atol=2e-6)
    ctx.close()
    table.close()


def test_c5_batched_full_size_chain_with_preset_table():
    """Preset C5 as one chained batched step: dart_draft_forward_batched over 16 ragged sequences
    -> dart_topk over the 128 logit rows -> dart_tree_prune over the 16 sequences with the
    2^20-context trigram table.  Top-k and pruning are checked for every row and every tree on
    the inputs those stages saw; the forward against the oracle on the shortest, the median and
    the longest sequence (a full fp64 forward of all 16 would take minutes)."""
    import torch
    import paper_2601_19278_amd as dart
    from dart_synth.tensors import make_ragged_lengths
    cfg = ds.get_config("C5")
    B, K, k = cfg.batch, cfg.K, cfg.topk
    ctx, W = make_context(cfg, 9600)
    counts = ds.make_ngram_counts(cfg, 9601)
    table = dart.NgramTable(cfg.n_gram, counts.keys, counts.succ_ids, counts.succ_counts, 1e-9)
    model = NgramModel(cfg.n_gram, counts.keys, counts.succ_ids, counts.succ_counts, 1e-9)
    lens = make_ragged_lengths(cfg, 9602).tolist()
    hiddens = [ds.make_hidden(cfg, 9603 + b, n=lens[b]) for b in range(B)]
    devs = [hidden_to_device(cfg, h) for h in hiddens]
    tails = np.ascontiguousarray(counts.keys[1000:1000 + B].astype(np.int32))   # stored contexts
    logits = ctx.draft_forward_batched(devs, lens, [0] * B, K)
    ids, scores = ctx.topk(logits.view(B * K, cfg.vocab), k, 1e-9)
    params = dart.PruneParams(k=k, beam_w=cfg.beam_w, budget=cfg.budget)
    tree = table.tree_prune(ids.view(B, K, k), scores.view(B, K, k), torch.from_numpy(tails).cuda(), params)
    torch.cuda.synchronize()
    logits, ids, scores = logits.cpu().numpy(), ids.cpu().numpy(), scores.cpu().numpy()
    tokens, parents, mask, n_nodes = [t.cpu().numpy() for t in tree]
    tol = dict(atol=2e-2, rtol=1e-2)
    order = np.argsort(lens)
    for b in (int(order[0]), int(order[B // 2]), int(order[-1])):
        ok, msg = logits_close(logits[b], odf.draft_forward(cfg, W, hiddens[b], K), **tol)
        assert ok, f"sequence {b} (n={lens[b]}): {msg}"
    ref_ids, ref_scores = otk.topk_rows(logits.reshape(B * K, cfg.vocab), k, 1e-9)
    np.testing.assert_array_equal(ids, ref_ids)
    np.testing.assert_allclose(scores, ref_scores, rtol=0, atol=1e-5)
    for b in range(B):
        ref = otp.tree_prune(ids.reshape(B, K, k)[b], scores.reshape(B, K, k)[b], tails[b], model,
                             otp.PruneParams(k=k, beam_w=cfg.beam_w, budget=cfg.budget))
        assert int(n_nodes[b]) == ref.n_nodes, b
        np.testing.assert_array_equal(tokens[b], ref.tokens)
        np.testing.assert_array_equal(parents[b], ref.parents)
        np.testing.assert_array_equal(mask[b], ref.mask)
    ctx.close()
    table.close()


def test_step_captured_in_a_hip_graph_replays_identically():
    """The hot calls enqueue kernels only (no allocation, no synchronisation, no host-side copies), so a
    whole step can be captured into a HIP graph; every replay, with eager steps and synchronisations
    in between, must reproduce the eager result bit for bit."""
    import torch
    import paper_2601_19278_amd as dart
    cfg = ds.scaled_config("C2", d=512, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn=1536, vocab=40007,
                           ctx=200, K=8)
    ctx, W = make_context(cfg, 9700)
    counts = ds.make_ngram_counts(cfg, 9701)
    table = dart.NgramTable(cfg.n_gram, counts.keys, counts.succ_ids, counts.succ_counts, 1e-9)
    h = hidden_to_device(cfg, ds.make_hidden(cfg, 9702))
    n, K, k = cfg.ctx, cfg.K, cfg.topk
    dev = h.device
    tk = (torch.empty((K, k), dtype=torch.int32, device=dev), torch.empty((K, k), dtype=torch.float32, device=dev))
    tree = (torch.empty((1, cfg.budget), dtype=torch.int32, device=dev),
            torch.empty((1, cfg.budget), dtype=torch.int32, device=dev),
            torch.empty((1, cfg.budget, cfg.budget), dtype=torch.uint8, device=dev),
            torch.empty((1,), dtype=torch.int32, device=dev))
    tail = torch.from_numpy(counts.keys[5].astype(np.int32)).cuda()[None]
    params = dart.PruneParams(k=k, beam_w=cfg.beam_w, budget=cfg.budget)

    def step():
        ctx.draft_forward_topk(h, n, K, k, 1e-9, n_cached=n - 3, out=tk)
        table.tree_prune(tk[0][None], tk[1][None], tail, params, out=tree)

    ctx.draft_forward(h, n, K)                      # fills the K/V cache (and loads every kernel)
    step()
    torch.cuda.synchronize()
    eager = [t.clone() for t in (*tk, *tree)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for i in range(4):
        for t in (*tk, *tree):
            t.zero_()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(eager, (*tk, *tree)):
            assert torch.equal(a, b), i
        step()                                      # eager work between the replays
        torch.cuda.synchronize()
    ctx.close()
    table.close()
