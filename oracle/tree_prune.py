"""Oracle: continuity-aware tree pruning (Alg. 1; constants and Combine in App. D).

`tree_prune` takes the algorithm's steps in the paper's order: K levels of beam
expansion, every expansion added to the global tree T before the beam cut, the
beam cut to the w best, and finally the theta best nodes of T.  `enumerate_tree`
is an independent second routine that scores *every* path of the full k-ary tree
by walking it from the root; it gives the expected answer whenever the beam never
cuts (w >= k^(K-1)).

Arithmetic that decides the tree is fixed in fp32, one rounding per operation, in
the literal order of the Combine formula:

    inc   = ((w_logit * s_logit) + (w_ng * s_ng)) * w_level
    score = parent_score + inc
    w_logit = fp32(decay^level), w_level = fp32((level+1)^-pow), level 0-based.

Ordering rules (the paper leaves ties open): beam cut by (score desc, creation
index asc) where creation = beam_rank * k + candidate_rank; global cut by (score
desc, level asc, creation asc).  Output order: root first, then level-major, and
within a level by (score desc, creation asc); parents therefore precede children.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np

f32 = np.float32


@dataclass
class PruneParams:
    k: int
    beam_w: int
    budget: int                 # nodes including the root; theta = budget - 1
    w_ng: float = 0.5
    logit_decay: float = 0.9
    level_pow: float = 0.7
    eps: float = 1e-9


@dataclass
class Tree:
    tokens: np.ndarray          # int32 [budget], -1 beyond n_nodes
    parents: np.ndarray         # int32 [budget], -1 for the root and beyond n_nodes
    mask: np.ndarray            # uint8 [budget][budget], mask[i][j]=1 iff j is i or an ancestor of i
    n_nodes: int
    scores: np.ndarray          # float32 [budget] path scores (root 0), for inspection
    levels: np.ndarray          # int32 [budget] (root -1)


def level_weights(params: PruneParams, level: int):
    wl = f32(math.pow(float(f32(params.logit_decay)), level))
    wv = f32(math.pow(level + 1.0, -float(f32(params.level_pow))))
    return wl, wv


def combine(params: PruneParams, level: int, s_logit, s_ng) -> np.float32:
    """Score increment of one edge, fp32, no fused multiply-add."""
    wl, wv = level_weights(params, level)
    a = f32(wl * f32(s_logit))
    b = f32(f32(params.w_ng) * f32(s_ng))
    return f32(f32(a + b) * wv)


def _context(ctx_tail, path_tokens, n_gram: int):
    seq = [int(t) for t in ctx_tail] + [int(t) for t in path_tokens]
    return tuple(seq[len(seq) - (n_gram - 1):])


def tree_prune(ids: np.ndarray, scores: np.ndarray, ctx_tail, ngram, params: PruneParams) -> Tree:
    """Alg. 1 for one sequence.  ids/scores: [K][>=k] candidates per level, best first."""
    K, k, w = ids.shape[0], params.k, params.beam_w
    theta = params.budget - 1
    root = dict(path=[], score=f32(0.0), parent=None, level=-1)
    beam = [root]                                          # C: (sequence, score)
    tree = []                                              # T
    for L in range(K):
        expanded = []
        for b, entry in enumerate(beam):
            row = ngram.lookup(_context(ctx_tail, entry["path"], ngram.n_gram))
            for c in range(k):
                t = int(ids[L, c])
                inc = combine(params, L, scores[L, c], ngram.score(row, t))
                node = dict(path=entry["path"] + [t], score=f32(entry["score"] + inc),
                            parent=None if entry is root else entry, token=t, level=L,
                            creation=b * k + c)
                expanded.append(node)
                tree.append(node)
        expanded.sort(key=lambda nd: (-float(nd["score"]), nd["creation"]))
        beam = expanded[: min(w, len(expanded))]
    tree.sort(key=lambda nd: (-float(nd["score"]), nd["level"], nd["creation"]))
    selected = tree[: min(theta, len(tree))]
    return _emit(selected, ctx_tail, params.budget)


def _emit(selected, ctx_tail, budget: int) -> Tree:
    selected = sorted(selected, key=lambda nd: (nd["level"], -float(nd["score"]), nd["creation"]))
    index = {id(nd): i + 1 for i, nd in enumerate(selected)}
    tokens = np.full(budget, -1, dtype=np.int32)
    parents = np.full(budget, -1, dtype=np.int32)
    mask = np.zeros((budget, budget), dtype=np.uint8)
    sc = np.zeros(budget, dtype=np.float32)
    lv = np.full(budget, -1, dtype=np.int32)
    tokens[0] = int(ctx_tail[-1])
    mask[0, 0] = 1
    for nd in selected:
        i = index[id(nd)]
        p = 0 if nd["parent"] is None else index[id(nd["parent"])]   # KeyError = not ancestor-closed
        tokens[i], parents[i], sc[i], lv[i] = nd["token"], p, nd["score"], nd["level"]
        mask[i] = mask[p]
        mask[i, i] = 1
    return Tree(tokens, parents, mask, 1 + len(selected), sc, lv)


def enumerate_tree(ids: np.ndarray, scores: np.ndarray, ctx_tail, ngram, params: PruneParams):
    """Every path of the full k-ary tree with its score: list of (path tuple, score).

    Each path is scored on its own by walking from the root and re-querying the
    N-gram model for every edge; nothing is shared with `tree_prune`'s loop.
    """
    K, k = ids.shape[0], params.k
    out = []

    def path_score(path_idx):
        s = f32(0.0)
        toks = []
        for L, c in enumerate(path_idx):
            row = ngram.lookup(_context(ctx_tail, toks, ngram.n_gram))
            t = int(ids[L, c])
            s = f32(s + combine(params, L, scores[L, c], ngram.score(row, t)))
            toks.append(t)
        return tuple(toks), s

    def rec(prefix):
        if prefix:
            out.append(path_score(prefix))
        if len(prefix) < K:
            for c in range(k):
                rec(prefix + [c])

    rec([])
    return out


def tree_paths(tree: Tree):
    """Root-to-node token paths (root excluded) and scores of an emitted tree."""
    paths = []
    for i in range(1, tree.n_nodes):
        toks, j = [], i
        while j != 0:
            toks.append(int(tree.tokens[j]))
            j = int(tree.parents[j])
        paths.append((tuple(reversed(toks)), f32(tree.scores[i])))
    return paths
