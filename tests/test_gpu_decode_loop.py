"""GPU parity over several draft-verify iterations in a row, the way decoding drives the library
(paper Sec. 2.1, Fig. 3): draft forward on the prefix with the rows of earlier iterations cached,
top-k, tree pruning, the greedy acceptance walk against a (synthetic) target, then the accepted
tokens extend the prefix by tau + 1 rows and the target's next token becomes the next root.
Every stage of every iteration is compared with the oracle on the inputs that stage saw; the
oracle recomputes each forward from scratch, so the evolving n_cached is what is under test."""
import numpy as np
import pytest

import dart_synth as ds
from oracle import draft_forward as odf, topk as otk, tree_prune as otp, verify as ovf
from oracle.ngram import NgramModel
from util_gpu import hidden_to_device, logits_close, make_context

pytestmark = pytest.mark.gpu


def _synthetic_target(rng, tokens, parents, n_nodes, vocab, agree):
    """Stand-in for the target's arg-max token after every tree node: with probability `agree`
    the token of one of the node's children (so that the walk goes on), else a random token."""
    out = rng.integers(0, vocab, size=tokens.shape[0]).astype(np.int32)
    for i in range(n_nodes):
        kids = [j for j in range(n_nodes) if parents[j] == i]
        if kids and rng.random() < agree:
            out[i] = tokens[kids[int(rng.integers(0, len(kids)))]]
    return out


def _step_checks(cfg, model, params, logits, ref_logits, ids, scores, tree, tail, tol):
    ok, msg = logits_close(logits, ref_logits, **tol)
    assert ok, msg
    ref_ids, ref_scores = otk.topk_rows(logits, cfg.topk, 1e-9)
    np.testing.assert_array_equal(ids, ref_ids)
    np.testing.assert_allclose(scores, ref_scores, rtol=0, atol=1e-5)
    tokens, parents, mask, n_nodes = tree
    ref = otp.tree_prune(ids, scores, tail, model, params)
    assert int(n_nodes) == ref.n_nodes
    np.testing.assert_array_equal(tokens, ref.tokens)
    np.testing.assert_array_equal(parents, ref.parents)
    np.testing.assert_array_equal(mask, ref.mask)
    return ref


@pytest.mark.parametrize("name,tol", [("C1", dict(atol=2e-4, rtol=2e-4)),
                                      ("bf16", dict(atol=2e-2, rtol=1e-2))])
def test_single_sequence_decode_loop(name, tol):
    import torch
    import paper_2601_19278_amd as dart
    cfg = ds.get_config("C1") if name == "C1" else ds.scaled_config(
        "C2", d=256, n_q_heads=4, n_kv_heads=2, head_dim=128, ffn=512, vocab=1000, ctx=120, K=6,
        topk=4, beam_w=6, budget=20, n_gram=2, n_keys=512, succ_per_key=8)
    ctx, W = make_context(cfg, 7100)
    counts = ds.make_ngram_counts(cfg, 7101)
    table = dart.NgramTable(cfg.n_gram, counts.keys, counts.succ_ids, counts.succ_counts, 1e-9)
    model = NgramModel(cfg.n_gram, counts.keys, counts.succ_ids, counts.succ_counts, 1e-9)
    gp = dart.PruneParams(k=cfg.topk, beam_w=cfg.beam_w, budget=cfg.budget)
    op = otp.PruneParams(k=cfg.topk, beam_w=cfg.beam_w, budget=cfg.budget)
    hidden = ds.make_hidden(cfg, 7102)              # the target's hidden states, position by position
    h_dev = hidden_to_device(cfg, hidden)
    rng = np.random.default_rng(7103)
    n = cfg.ctx // 3
    seq = rng.integers(0, cfg.vocab, size=n + 1).astype(np.int32).tolist()   # prefix + root t_{n+1}
    cached, taus = 0, []
    while n + cfg.K + 1 <= cfg.ctx:
        tail = np.asarray(seq[-(cfg.n_gram - 1):], dtype=np.int32)
        if name == "C1":
            logits = ctx.draft_forward(h_dev, n, cfg.K, n_cached=cached)
            ids, scores = ctx.topk(logits, cfg.topk, 1e-9)
        else:       # bf16: forward and top-k as one call (the LM head selects its candidates itself)
            logits = torch.empty((cfg.K, cfg.vocab), dtype=torch.float32, device="cuda")
            ids, scores = ctx.draft_forward_topk(h_dev, n, cfg.K, cfg.topk, 1e-9, n_cached=cached,
                                                 logits_out=logits)
        tree_dev = table.tree_prune(ids, scores, torch.from_numpy(tail).cuda(), gp)
        tree = [t.cpu().numpy() for t in tree_dev]
        ref_tree = _step_checks(cfg, model, op, logits.cpu().numpy(),
                                odf.draft_forward(cfg, W, hidden[:n], cfg.K), ids.cpu().numpy(),
                                scores.cpu().numpy(), tree, tail, tol)
        target_next = _synthetic_target(rng, ref_tree.tokens, ref_tree.parents, ref_tree.n_nodes,
                                        cfg.vocab, agree=0.7)
        tk, pr, _, nn = tree_dev
        pos, path, n_acc, nxt = dart.tree_verify_greedy(
            tk.reshape(1, -1), pr.reshape(1, -1), nn.reshape(1),
            ctx_len=torch.tensor([n], dtype=torch.int32, device="cuda"),
            target_next=torch.from_numpy(target_next).cuda().reshape(1, -1))
        ref_pos = ovf.tree_positions(ref_tree.parents, ref_tree.n_nodes)
        ref_path, ref_next = ovf.accept_greedy(ref_tree.tokens, ref_tree.parents, ref_tree.n_nodes,
                                               target_next)
        np.testing.assert_array_equal(pos.cpu().numpy()[0][: ref_tree.n_nodes], ref_pos + n)
        tau = int(n_acc.cpu()[0])
        assert tau == len(ref_path) - 1 and int(nxt.cpu()[0]) == ref_next
        np.testing.assert_array_equal(path.cpu().numpy()[0][: tau + 1], ref_path)
        # the root and the accepted tokens now have hidden states; the target's token is the new root
        seq += [int(ref_tree.tokens[i]) for i in ref_path[1:]] + [ref_next]
        cached, n = n, n + 1 + tau
        taus.append(tau)
    assert len(taus) >= 4 and max(taus) >= 2 and min(taus) < max(taus), taus
    ctx.close()
    table.close()


def test_batched_decode_loop_with_diverging_lengths():
    """Three sequences advance by different amounts per iteration (their own tau), so the batched
    call sees ragged lengths and per-sequence n_cached that drift apart."""
    import torch
    import paper_2601_19278_amd as dart
    B = 3
    cfg = ds.scaled_config("C2", d=256, n_q_heads=4, n_kv_heads=2, head_dim=128, ffn=512, vocab=1024,
                           ctx=110, K=5, topk=4, beam_w=5, budget=16, n_gram=2, n_keys=512,
                           succ_per_key=8, batch=B)
    ctx, W = make_context(cfg, 7200)
    counts = ds.make_ngram_counts(cfg, 7201)
    table = dart.NgramTable(cfg.n_gram, counts.keys, counts.succ_ids, counts.succ_counts, 1e-9)
    model = NgramModel(cfg.n_gram, counts.keys, counts.succ_ids, counts.succ_counts, 1e-9)
    gp = dart.PruneParams(k=cfg.topk, beam_w=cfg.beam_w, budget=cfg.budget)
    op = otp.PruneParams(k=cfg.topk, beam_w=cfg.beam_w, budget=cfg.budget)
    hiddens = [ds.make_hidden(cfg, 7210 + b) for b in range(B)]
    devs = [hidden_to_device(cfg, h) for h in hiddens]
    rng = np.random.default_rng(7203)
    lens = [20, 41, 33]
    seqs = [rng.integers(0, cfg.vocab, size=lens[b] + 1).astype(np.int32).tolist() for b in range(B)]
    cached = [0] * B
    tol = dict(atol=2e-2, rtol=1e-2)
    for it in range(8):
        if max(lens) + cfg.K + 1 > cfg.ctx:
            break
        tails = np.stack([np.asarray(s[-(cfg.n_gram - 1):], dtype=np.int32) for s in seqs])
        logits = torch.empty((B, cfg.K, cfg.vocab), dtype=torch.float32, device="cuda")
        if it % 2 == 0:
            ctx.draft_forward_batched(devs, lens, cached, cfg.K, out=logits)
            ids, scores = ctx.topk(logits.reshape(B * cfg.K, -1), cfg.topk, 1e-9)
            ids, scores = ids.reshape(B, cfg.K, -1), scores.reshape(B, cfg.K, -1)
        else:       # every other iteration through the combined call
            ids, scores = ctx.draft_forward_topk_batched(devs, lens, cached, cfg.K, cfg.topk, 1e-9,
                                                         logits_out=logits)
        tk, pr, mk, nn = table.tree_prune(ids, scores, torch.from_numpy(tails).cuda(), gp)
        refs, targets = [], []
        for b in range(B):
            refs.append(_step_checks(cfg, model, op, logits[b].cpu().numpy(),
                                     odf.draft_forward(cfg, W, hiddens[b][: lens[b]], cfg.K),
                                     ids[b].cpu().numpy(), scores[b].cpu().numpy(),
                                     [t[b].cpu().numpy() for t in (tk, pr, mk, nn)], tails[b], tol))
            targets.append(_synthetic_target(rng, refs[b].tokens, refs[b].parents, refs[b].n_nodes,
                                             cfg.vocab, agree=0.5 + 0.2 * b))
        pos, path, n_acc, nxt = dart.tree_verify_greedy(
            tk, pr, nn, ctx_len=torch.tensor(lens, dtype=torch.int32, device="cuda"),
            target_next=torch.from_numpy(np.stack(targets)).cuda())
        for b in range(B):
            ref_path, ref_next = ovf.accept_greedy(refs[b].tokens, refs[b].parents, refs[b].n_nodes,
                                                   targets[b])
            tau = int(n_acc.cpu()[b])
            assert tau == len(ref_path) - 1 and int(nxt.cpu()[b]) == ref_next
            np.testing.assert_array_equal(path.cpu().numpy()[b][: tau + 1], ref_path)
            seqs[b] += [int(refs[b].tokens[i]) for i in ref_path[1:]] + [ref_next]
            cached[b], lens[b] = lens[b], lens[b] + 1 + tau
    assert it >= 4 and len(set(lens)) == B
    ctx.close()
    table.close()
