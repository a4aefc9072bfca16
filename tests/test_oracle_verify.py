"""Pins for the oracle's verification glue (tree positions, greedy acceptance walk): hand
trees, a chain (longest common prefix), brute force over all root-to-node paths, and planted
mistakes."""
import itertools

import numpy as np

import dart_synth as ds
from oracle import tree_prune as otp
from oracle import verify as ov
from oracle.ngram import NgramModel


def _random_tree(seed, K=6, k=4, w=5, budget=30):
    case = ds.make_prune_case(seed, vocab=500, K=K, k=k, n_gram=3, S=8)
    model = NgramModel(3, case.table.keys, case.table.succ_ids, case.table.succ_counts, 1e-9)
    return otp.tree_prune(case.ids, case.scores, case.ctx_tail, model,
                          otp.PruneParams(k=k, beam_w=w, budget=budget))


def test_hand_tree_positions_and_walk():
    # root(7) -> a(1) -> c(3) -> e(5)
    #         -> b(2) -> d(4)
    tokens = np.array([7, 1, 2, 3, 4, 5, -1, -1], np.int32)
    parents = np.array([-1, 0, 0, 1, 2, 3, -1, -1], np.int32)
    assert ov.tree_positions(parents, 6).tolist() == [0, 1, 1, 2, 2, 3, -1, -1]
    # target continues 7 -> 1 -> 3 -> 9: accepts a, c; e (5) is rejected; bonus token 9
    tn = np.array([1, 3, 0, 9, 0, 0, 0, 0], np.int32)
    assert ov.accept_greedy(tokens, parents, 6, tn) == ([0, 1, 3], 9)
    # target continues 7 -> 2 -> 4 -> 8: the other branch, to its leaf
    tn = np.array([2, 0, 4, 0, 8, 0, 0, 0], np.int32)
    assert ov.accept_greedy(tokens, parents, 6, tn) == ([0, 2, 4], 8)
    # nothing matches: only the root, bonus token = target's token after the root
    tn = np.array([6, 3, 4, 5, 0, 0, 0, 0], np.int32)
    assert ov.accept_greedy(tokens, parents, 6, tn) == ([0], 6)


def test_chain_is_longest_common_prefix():
    draft = [11, 12, 13, 14, 15]
    tokens = np.array([99] + draft, np.int32)
    parents = np.array([-1, 0, 1, 2, 3, 4], np.int32)
    for m in range(6):                       # target agrees with the first m drafted tokens
        truth = draft[:m] + [77] * (6 - m)   # target's token after node i is truth[i]
        path, nxt = ov.accept_greedy(tokens, parents, 6, np.array(truth, np.int32))
        assert path == list(range(m + 1)) and nxt == 77


def test_walk_equals_brute_force_over_all_paths():
    """The accepted path is the deepest root-to-node path all of whose edges match."""
    rng = np.random.default_rng(5)
    for seed in range(30):
        tr = _random_tree(100 + seed)
        n = tr.n_nodes
        tn = rng.integers(0, 500, size=len(tr.tokens)).astype(np.int32)
        # make some edges match on purpose: the target repeats a random child's token
        for i in range(n):
            kids = [c for c in range(n) if tr.parents[c] == i]
            if kids and rng.random() < 0.7:
                tn[i] = tr.tokens[kids[rng.integers(len(kids))]]
        best = [0]
        for i in range(n):
            path, j = [], i
            while j >= 0:
                path.append(j)
                j = int(tr.parents[j])
            path.reverse()
            if all(tr.tokens[c] == tn[p] for p, c in zip(path[:-1], path[1:])) and len(path) > len(best):
                best = path
        path, nxt = ov.accept_greedy(tr.tokens, tr.parents, n, tn)
        assert path == best and nxt == tn[best[-1]]
        depth = ov.tree_positions(tr.parents, n)
        assert (depth[:n] == tr.levels[:n] + 1).all() and (depth[n:] == -1).all()
        assert (depth[:n] == tr.mask[:n].sum(axis=1) - 1).all()      # ancestors incl. self, minus self


def test_planted_mistakes_are_caught():
    tokens = np.array([7, 1, 2, 3], np.int32)
    parents = np.array([-1, 0, 0, 1], np.int32)
    tn = np.array([2, 3, 3, 0], np.int32)
    # comparing with the child's own target token instead of the parent's would accept node 1
    assert ov.accept_greedy(tokens, parents, 4, tn) == ([0, 2], 3)
    # ignoring the parent link would accept node 3 (token 3 == tn[2]) although it hangs under node 1
    assert ov.accept_greedy(tokens, parents, 4, tn)[0] != [0, 2, 3]
