"""Pins for the oracle's N-gram model and tree pruning (Alg. 1, App. C.2, App. D)."""
import heapq
import math
import os

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import dart_synth as ds
from oracle.ngram import NgramModel
from oracle import tree_prune as otp
from oracle.tree_prune import PruneParams

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "prune_hand_example.txt")
f32 = np.float32


# ------------------------------------------------------------------ N-gram model
def test_ngram_probabilities_are_count_ratios():
    keys = np.array([[5, 6], [6, 7]], dtype=np.int32)
    ids = np.array([[10, 11, -1], [12, 13, 14]], dtype=np.int32)
    cnt = np.array([[3, 1, 0], [1, 1, 2]], dtype=np.int32)
    ng = NgramModel(3, keys, ids, cnt, 1e-9)
    row = ng.lookup((5, 6))
    assert set(row) == {10, 11}
    np.testing.assert_allclose(row[10], math.log(0.75), rtol=1e-6)
    np.testing.assert_allclose(row[11], math.log(0.25), rtol=1e-6)
    np.testing.assert_allclose(ng.score(row, 99), math.log(1e-9), rtol=1e-6)   # unseen successor
    assert ng.lookup((6, 5)) is None                                           # order matters
    np.testing.assert_allclose(ng.score(None, 10), math.log(1e-9), rtol=1e-6)  # unseen context
    single = NgramModel(2, np.array([[4]], np.int32), np.array([[9]], np.int32),
                        np.array([[7]], np.int32), 1e-9)
    assert single.lookup((4,))[9] == 0.0                                       # Pr=1 clamps to 0


# ------------------------------------------------------------------ hand example
def _hand_case():
    A, B, C, D, ROOT, X = 1, 2, 3, 4, 0, 9
    ids = np.array([[A, B], [C, D]], dtype=np.int32)
    scores = np.log(np.array([[0.6, 0.3], [0.5, 0.2]])).astype(np.float32)
    keys = np.array([[ROOT], [A], [B]], dtype=np.int32)
    succ = np.array([[A, B, X], [C, X, -1], [C, D, -1]], dtype=np.int32)
    cnt = np.array([[2, 1, 1], [4, 1, 0], [1, 9, 0]], dtype=np.int32)
    names = {(A,): "A", (B,): "B", (A, C): "AC", (A, D): "AD", (B, C): "BC", (B, D): "BD"}
    return ids, scores, np.array([ROOT], np.int32), NgramModel(2, keys, succ, cnt, 1e-9), names


@pytest.mark.parametrize("variant,w_ng", [("ngram", 0.5), ("nongram", 0.0)])
def test_hand_derived_example(variant, w_ng):
    expected = {}
    for line in open(GOLDEN):
        if line.startswith(variant + " "):
            _, path, score, kept = line.split()
            expected[path] = (float(score), kept == "1")
    assert len(expected) == 6
    ids, scores, tail, ng, names = _hand_case()
    full = otp.tree_prune(ids, scores, tail, ng, PruneParams(k=2, beam_w=4, budget=7, w_ng=w_ng))
    got = {names[p]: float(s) for p, s in otp.tree_paths(full)}
    assert set(got) == set(expected)
    for path, (score, _) in expected.items():
        assert abs(got[path] - score) < 6e-5, (path, got[path], score)
    top4 = otp.tree_prune(ids, scores, tail, ng, PruneParams(k=2, beam_w=4, budget=5, w_ng=w_ng))
    kept = {names[p] for p, _ in otp.tree_paths(top4)}
    assert kept == {p for p, (_, keep) in expected.items() if keep}


# ------------------------------------------------------------------ back-off (optional reading)
def _backoff_hand_case(with_backoff):
    A, B, C, D, P, R, X = 1, 2, 3, 4, 7, 0, 9
    ids = np.array([[A, B], [C, D]], dtype=np.int32)
    scores = np.log(np.array([[0.6, 0.3], [0.5, 0.2]])).astype(np.float32)
    keys = np.array([[P, R], [R, B]], dtype=np.int32)
    succ = np.array([[A, B, X], [C, D, -1]], dtype=np.int32)
    cnt = np.array([[2, 1, 1], [1, 9, 0]], dtype=np.int32)
    lower = NgramModel(2, np.array([[A]], np.int32), np.array([[C, X]], np.int32),
                       np.array([[4, 1]], np.int32), 1e-9, discount=0.4) if with_backoff else None
    names = {(A,): "A", (B,): "B", (A, C): "AC", (A, D): "AD", (B, C): "BC", (B, D): "BD"}
    return ids, scores, np.array([P, R], np.int32), NgramModel(3, keys, succ, cnt, 1e-9, backoff=lower), names


@pytest.mark.parametrize("variant", ["tri_plain", "tri_backoff"])
def test_hand_derived_backoff_example(variant):
    expected = {}
    for line in open(GOLDEN):
        if line.startswith(variant + " "):
            _, path, score, kept = line.split()
            expected[path] = (float(score), kept == "1")
    assert len(expected) == 6
    ids, scores, tail, ng, names = _backoff_hand_case(variant == "tri_backoff")
    full = otp.tree_prune(ids, scores, tail, ng, PruneParams(k=2, beam_w=4, budget=7))
    got = {names[p]: float(s) for p, s in otp.tree_paths(full)}
    for path, (score, _) in expected.items():
        assert abs(got[path] - score) < 6e-5, (path, got[path], score)
    top4 = otp.tree_prune(ids, scores, tail, ng, PruneParams(k=2, beam_w=4, budget=5))
    assert {names[p] for p, _ in otp.tree_paths(top4)} == {p for p, (_, keep) in expected.items() if keep}


def test_backoff_scores_and_precedence():
    keys = np.array([[5, 6]], dtype=np.int32)
    main_ids, main_cnt = np.array([[10, 11]], np.int32), np.array([[3, 1]], np.int32)
    low = NgramModel(2, np.array([[6], [8]], np.int32), np.array([[10, 12], [13, -1]], np.int32),
                     np.array([[1, 3], [5, 0]], np.int32), 1e-9, discount=0.25)
    ng = NgramModel(3, keys, main_ids, main_cnt, 1e-9, backoff=low)
    row = ng.lookup((5, 6))                       # stored: never backs off, although (6) exists below
    np.testing.assert_allclose(row[10], math.log(0.75), rtol=1e-6)
    assert 12 not in row and ng.score(row, 12) == ng.miss
    row = ng.lookup((9, 6))                       # unseen: the context without its oldest token
    np.testing.assert_allclose(row[10], math.log(0.25 * 0.25), rtol=1e-6)
    np.testing.assert_allclose(row[12], math.log(0.25 * 0.75), rtol=1e-6)
    row = ng.lookup((6, 8))                       # drops the OLDEST token: (8), not (6)
    np.testing.assert_allclose(row[13], math.log(0.25), rtol=1e-6)
    assert ng.lookup((1, 2)) is None              # unseen in both: log eps as before
    plain = NgramModel(3, keys, main_ids, main_cnt, 1e-9)
    assert plain.lookup((9, 6)) is None           # off by default


@pytest.mark.parametrize("seed", range(6))
def test_empty_trigram_table_with_undiscounted_backoff_is_the_bigram_model(seed):
    """Every trigram lookup misses and falls to the bigram table with alpha = 1: the tree must be
    the one a plain bigram model gives for the same candidates (the context loses its oldest
    token, nothing else changes)."""
    K, k = 4, 3
    pc = ds.make_prune_case(300 + seed, vocab=64, K=K, k=k, n_gram=2, S=8, n_filler_keys=8)
    bigram = NgramModel(2, pc.table.keys, pc.table.succ_ids, pc.table.succ_counts, 1e-9)
    empty3 = NgramModel(3, np.zeros((0, 2), np.int32), np.zeros((0, 8), np.int32),
                        np.zeros((0, 8), np.int32), 1e-9,
                        backoff=NgramModel(2, pc.table.keys, pc.table.succ_ids, pc.table.succ_counts, 1e-9))
    tail3 = np.array([17, int(pc.ctx_tail[0])], np.int32)
    for w, budget in ((2, 9), (27, 30)):
        params = PruneParams(k=k, beam_w=w, budget=budget)
        a = otp.tree_prune(pc.ids, pc.scores, pc.ctx_tail, bigram, params)
        b = otp.tree_prune(pc.ids, pc.scores, tail3, empty3, params)
        np.testing.assert_array_equal(a.tokens, b.tokens)
        np.testing.assert_array_equal(a.parents, b.parents)
        np.testing.assert_array_equal(a.scores, b.scores)
        assert a.n_nodes == b.n_nodes


@pytest.mark.parametrize("seed", range(4))
def test_backoff_keeps_the_invariants_and_is_idle_when_every_context_is_stored(seed):
    K, k = 4, 3
    pc, ng = _case(400 + seed, K=K, k=k, n_gram=3)
    lowc = ds.make_prune_case(500 + seed, vocab=64, K=K, k=k, n_gram=2, S=8, n_filler_keys=40)
    # bigram rows for the trigram case's own candidates, so that back-off really hits
    low_keys = np.unique(np.concatenate([pc.ids[:-1].ravel(), pc.ctx_tail[-1:]]))[:, None].astype(np.int32)
    low_ids = np.stack([np.resize(np.random.default_rng(seed + i).permutation(pc.ids[min(K - 1, 1 + i % (K - 1))]), 8)
                        for i in range(low_keys.shape[0])]).astype(np.int32)
    low_ids[:, k:] = -1
    low_cnt = (low_ids >= 0).astype(np.int32) * np.arange(1, 9, dtype=np.int32)[None, :]
    low = NgramModel(2, low_keys, low_ids, low_cnt, 1e-9, discount=0.4)
    both = NgramModel(3, pc.table.keys, pc.table.succ_ids, pc.table.succ_counts, 1e-9, backoff=low)
    params = PruneParams(k=k, beam_w=4, budget=20)
    tree = otp.tree_prune(pc.ids, pc.scores, pc.ctx_tail, both, params)
    _check_invariants(tree, pc, both, params, K)
    plain = otp.tree_prune(pc.ids, pc.scores, pc.ctx_tail, ng, params)
    assert not np.array_equal(tree.scores, plain.scores)      # back-off changed some score
    # a main table that stores every context the candidates can present never consults it
    ctxs = {tuple(int(t) for t in pc.ctx_tail)} | {(int(pc.ctx_tail[1]), int(t)) for t in pc.ids[0]}
    for L in range(2, K):
        ctxs |= {(int(a), int(t)) for a in pc.ids[L - 2] for t in pc.ids[L - 1]}
    have = {tuple(int(t) for t in key) for key in pc.table.keys}
    extra = sorted(ctxs - have)
    keys2 = np.concatenate([pc.table.keys, np.array(extra, np.int32).reshape(-1, 2)])
    ids2 = np.concatenate([pc.table.succ_ids, np.full((len(extra), 8), -1, np.int32)])
    cnt2 = np.concatenate([pc.table.succ_counts, np.zeros((len(extra), 8), np.int32)])
    ids2[len(pc.table.keys):, 0], cnt2[len(pc.table.keys):, 0] = 63, 1      # a successor no level proposes
    full_plain = NgramModel(3, keys2, ids2, cnt2, 1e-9)
    full_both = NgramModel(3, keys2, ids2, cnt2, 1e-9, backoff=low)
    a = otp.tree_prune(pc.ids, pc.scores, pc.ctx_tail, full_plain, params)
    b = otp.tree_prune(pc.ids, pc.scores, pc.ctx_tail, full_both, params)
    np.testing.assert_array_equal(a.tokens, b.tokens)
    np.testing.assert_array_equal(a.scores, b.scores)


def test_combine_is_the_printed_formula_in_fp32_without_fma():
    p = PruneParams(k=1, beam_w=1, budget=2)
    s_logit, s_ng = f32(-1.2345678), f32(-7.654321)
    for level in range(8):
        wl = f32(f32(0.9).astype(np.float64) ** level)
        wv = f32((level + 1.0) ** -f32(0.7).astype(np.float64))
        want = f32(f32(f32(wl * s_logit) + f32(f32(0.5) * s_ng)) * wv)
        assert otp.combine(p, level, s_logit, s_ng) == want
    assert otp.level_weights(p, 0) == (f32(1.0), f32(1.0))
    np.testing.assert_allclose(otp.level_weights(p, 1), (0.9, 2 ** -0.7), rtol=1e-6)
    np.testing.assert_allclose(otp.level_weights(p, 7), (0.9 ** 7, 8 ** -0.7), rtol=1e-6)


# ------------------------------------------------------------------ helpers
def _case(seed, K=4, k=3, n_gram=3, S=8, vocab=64):
    pc = ds.make_prune_case(seed, vocab=vocab, K=K, k=k, n_gram=n_gram, S=S, n_filler_keys=8)
    ng = NgramModel(n_gram, pc.table.keys, pc.table.succ_ids, pc.table.succ_counts, 1e-9)
    return pc, ng


def _check_invariants(tree, pc, ng, params, K):
    """Structural invariants of any emitted tree, with N-gram continuity re-verified
    on every edge by rescoring each node's path from scratch."""
    n = tree.n_nodes
    assert tree.tokens[0] == pc.ctx_tail[-1] and tree.parents[0] == -1
    assert (tree.tokens[n:] == -1).all() and (tree.parents[n:] == -1).all()
    assert not tree.mask[n:].any() and not tree.mask[:, n:].any()
    level = {0: -1}
    for i in range(1, n):
        p = int(tree.parents[i])
        assert 0 <= p < i                                       # parents precede children
        level[i] = level[p] + 1
        assert level[i] == tree.levels[i] < K
        assert tree.tokens[i] in pc.ids[level[i], : params.k]   # token comes from its level
        assert tree.scores[i] <= tree.scores[p]                 # monotone along a path
    for i in range(1, n):
        for j in range(i + 1, n):
            if tree.parents[i] == tree.parents[j]:
                assert tree.tokens[i] != tree.tokens[j]         # siblings distinct
    for i in range(n):                                          # mask = ancestor closure
        anc, j = set(), i
        while j != -1:
            anc.add(j)
            j = int(tree.parents[j])
        assert set(np.nonzero(tree.mask[i])[0].tolist()) == anc
    order = [(tree.levels[i], -tree.scores[i]) for i in range(1, n)]
    assert order == sorted(order)                               # level-major, best first
    for path, score in otp.tree_paths(tree):                    # continuity on every edge
        s, toks = f32(0.0), []
        for L, t in enumerate(path):
            ctx = (list(pc.ctx_tail) + toks)[-(ng.n_gram - 1):]
            c = pc.ids[L].tolist().index(t)
            s = f32(s + otp.combine(params, L, pc.scores[L, c], ng.score(ng.lookup(ctx), t)))
            toks.append(t)
        assert s == score


def _no_ties(nodes):
    vals = sorted(float(s) for _, s in nodes)
    return all(a != b for a, b in zip(vals, vals[1:]))


# ------------------------------------------------------------------ exhaustive / best-first
@pytest.mark.parametrize("seed", range(12))
@pytest.mark.parametrize("n_gram", [2, 3])
def test_wide_beam_equals_exhaustive_enumeration(seed, n_gram):
    K, k = 4, 3
    pc, ng = _case(seed, K=K, k=k, n_gram=n_gram)
    for theta in (1, 5, 17, 40):
        params = PruneParams(k=k, beam_w=k ** (K - 1), budget=theta + 1)
        tree = otp.tree_prune(pc.ids, pc.scores, pc.ctx_tail, ng, params)
        every = otp.enumerate_tree(pc.ids, pc.scores, pc.ctx_tail, ng, params)
        assert len(every) == sum(k ** (L + 1) for L in range(K)) and _no_ties(every)
        best = sorted(every, key=lambda ps: -float(ps[1]))[:theta]
        assert sorted(otp.tree_paths(tree)) == sorted(best)
        _check_invariants(tree, pc, ng, params, K)


@pytest.mark.parametrize("seed", range(6))
def test_wide_beam_equals_best_first_search(seed):
    """Scores never increase along a path, so popping a max-heap of frontier nodes
    yields the global top-theta in order -- a third, independent construction."""
    K, k, theta = 4, 3, 25
    pc, ng = _case(100 + seed, K=K, k=k)
    params = PruneParams(k=k, beam_w=k ** (K - 1), budget=theta + 1)
    tree = otp.tree_prune(pc.ids, pc.scores, pc.ctx_tail, ng, params)

    def children(path, s):
        L = len(path)
        row = ng.lookup((list(pc.ctx_tail) + list(path))[-(ng.n_gram - 1):])
        for c in range(k):
            t = int(pc.ids[L, c])
            yield path + (t,), f32(s + otp.combine(params, L, pc.scores[L, c], ng.score(row, t)))

    heap = [(-float(s), p) for p, s in children((), f32(0.0))]
    heapq.heapify(heap)
    popped = []
    while heap and len(popped) < theta:
        neg, path = heapq.heappop(heap)
        popped.append((path, f32(-neg)))
        if len(path) < K:
            for p, s in children(path, f32(-neg)):
                heapq.heappush(heap, (-float(s), p))
    assert sorted(otp.tree_paths(tree)) == sorted(popped)


@pytest.mark.parametrize("seed", range(8))
@pytest.mark.parametrize("w", [1, 2, 4, 7])
def test_finite_beam_equals_its_set_definition_over_all_paths(seed, w):
    """Brute force for a beam that does cut: score every path of the full k-ary tree (the
    enumerator, itself pinned by the best-first search), then read Alg. 1 as sets -- the
    expansions of a level are the children of the previous level's beam, all of them enter T,
    the beam is the w best of them, and the tree is the theta best of T."""
    K, k = 4, 3
    pc, ng = _case(200 + seed, K=K, k=k)
    wide = PruneParams(k=k, beam_w=k ** (K - 1), budget=2)
    every = otp.enumerate_tree(pc.ids, pc.scores, pc.ctx_tail, ng, wide)
    assert _no_ties(every)
    for theta in (3, 11, 30):
        beam, T = {()}, []
        for L in range(K):
            level = [(p, sc) for p, sc in every if len(p) == L + 1 and p[:-1] in beam]
            T += level
            beam = {p for p, _ in sorted(level, key=lambda ps: -float(ps[1]))[:w]}
        best = sorted(T, key=lambda ps: -float(ps[1]))[:theta]
        tree = otp.tree_prune(pc.ids, pc.scores, pc.ctx_tail, ng,
                              PruneParams(k=k, beam_w=w, budget=theta + 1))
        assert sorted(otp.tree_paths(tree)) == sorted(best)


# ------------------------------------------------------------------ special cases
def test_k1_gives_the_argmax_chain():
    pc, ng = _case(7, K=5, k=3)
    for budget in (3, 6, 20):
        tree = otp.tree_prune(pc.ids, pc.scores, pc.ctx_tail, ng, PruneParams(k=1, beam_w=4, budget=budget))
        n = min(5, budget - 1)
        assert tree.n_nodes == n + 1
        assert tree.tokens[1: n + 1].tolist() == pc.ids[:n, 0].tolist()
        assert tree.parents[: n + 1].tolist() == [-1] + list(range(n))


def test_large_theta_and_wide_beam_return_the_full_tree():
    K, k = 3, 3
    pc, ng = _case(8, K=K, k=k)
    total = k + k * k + k ** 3
    params = PruneParams(k=k, beam_w=k ** (K - 1), budget=total + 10)
    tree = otp.tree_prune(pc.ids, pc.scores, pc.ctx_tail, ng, params)
    assert tree.n_nodes == total + 1
    assert [int((tree.levels == L).sum()) for L in range(K)] == [k, k * k, k ** 3]
    _check_invariants(tree, pc, ng, params, K)


def test_zero_ngram_weight_ignores_the_table_and_empty_table_keeps_levelwise_order():
    K, k = 4, 3
    pc, ng = _case(9, K=K, k=k)
    empty = NgramModel(3, np.zeros((0, 2), np.int32), np.zeros((0, 8), np.int32),
                       np.zeros((0, 8), np.int32), 1e-9)
    p0 = PruneParams(k=k, beam_w=4, budget=20, w_ng=0.0)
    a = otp.tree_prune(pc.ids, pc.scores, pc.ctx_tail, ng, p0)
    b = otp.tree_prune(pc.ids, pc.scores, pc.ctx_tail, empty, p0)
    np.testing.assert_array_equal(a.tokens, b.tokens)
    np.testing.assert_array_equal(a.parents, b.parents)
    np.testing.assert_array_equal(a.scores, b.scores)
    # empty table, w_ng > 0: each level gets one additive constant, so the complete tree
    # (no theta cut) has the same shape and within-level order as with w_ng = 0
    big = 3 + 3 * 4 * 3 + 10
    c = otp.tree_prune(pc.ids, pc.scores, pc.ctx_tail, empty, PruneParams(k=k, beam_w=4, budget=big))
    d = otp.tree_prune(pc.ids, pc.scores, pc.ctx_tail, empty, PruneParams(k=k, beam_w=4, budget=big, w_ng=0.0))
    np.testing.assert_array_equal(c.tokens, d.tokens)
    np.testing.assert_array_equal(c.parents, d.parents)


def test_beam_cut_nodes_stay_in_the_tree_as_leaves():
    """Alg. 1 adds every expansion to T before the beam is cut."""
    K, k = 3, 3
    pc, ng = _case(10, K=K, k=k)
    tree = otp.tree_prune(pc.ids, pc.scores, pc.ctx_tail, ng, PruneParams(k=k, beam_w=1, budget=100))
    # level sizes: k, then (1 beam) * k per level -> all 3K nodes kept
    assert tree.n_nodes == 1 + 3 * K
    for L in range(1, K):
        parents = {int(tree.parents[i]) for i in range(1, tree.n_nodes) if tree.levels[i] == L}
        assert len(parents) == 1                                 # only the single beam entry expands


def test_tie_breaks_shallower_then_creation_order():
    # all scores zero: every node ties; the cut must prefer shallow levels, then creation order
    ids = np.array([[3, 4], [5, 6], [7, 8]], dtype=np.int32)
    scores = np.zeros((3, 2), dtype=np.float32)
    empty = NgramModel(2, np.zeros((0, 1), np.int32), np.zeros((0, 4), np.int32),
                       np.zeros((0, 4), np.int32), 1e-9)
    tree = otp.tree_prune(ids, scores, np.array([1], np.int32), empty,
                          PruneParams(k=2, beam_w=2, budget=6, w_ng=0.0))
    assert tree.tokens[:6].tolist() == [1, 3, 4, 5, 6, 5]
    assert tree.parents[:6].tolist() == [-1, 0, 0, 1, 1, 2]


# ------------------------------------------------------------------ property test, finite beam
@settings(max_examples=60, deadline=None)
@given(seed=st.integers(0, 10_000), K=st.integers(1, 5), k=st.integers(1, 4), w=st.integers(1, 6),
       budget=st.integers(1, 30), n_gram=st.sampled_from([2, 3]))
def test_invariants_hold_for_any_beam(seed, K, k, w, budget, n_gram):
    pc, ng = _case(seed, K=K, k=k, n_gram=n_gram)
    params = PruneParams(k=k, beam_w=w, budget=budget)
    tree = otp.tree_prune(pc.ids, pc.scores, pc.ctx_tail, ng, params)
    sizes, beam = [], 1
    for _ in range(K):
        sizes.append(beam * k)
        beam = min(w, beam * k)
    assert tree.n_nodes == 1 + min(budget - 1, sum(sizes))
    _check_invariants(tree, pc, ng, params, K)
