"""Oracle: the N-gram continuity model g_n (Alg. 1 "s_ng", App. C.2, App. D).

A context (the previous N-1 tokens) maps to the list of successors seen after it,
with counts.  One context lookup serves every candidate of that context (the
single-traversal retrieval of App. C.2).  The score of candidate t is

    s_ng = log(Pr(t | context) + eps),   Pr = count(context, t) / sum of the
                                              context's stored counts,

and Pr = 0 (so s_ng = log eps) when the context or the successor is absent.  The
value is computed in fp64, rounded once to fp32 and clamped to <= 0.

Back-off (optional, off unless a lower-order model is given; the paper stores its
N-grams in a trie, App. C.2, and says nothing about contexts the trie has not seen):
a context that is absent from the table is looked up again without its oldest token
in a model of order N-1, whose successors then score

    s_ng = log(alpha * Pr_{N-1}(t | shorter context) + eps),

alpha being a fixed discount for the shorter context.  A context that IS stored never
backs off: its unseen successors keep log eps.  One level of back-off only.
"""
from __future__ import annotations

import math

import numpy as np


class NgramModel:
    def __init__(self, n_gram: int, keys: np.ndarray, succ_ids: np.ndarray,
                 succ_counts: np.ndarray, eps: float, backoff: "NgramModel | None" = None,
                 discount: float = 1.0):
        """backoff: a model of order n_gram - 1 consulted for contexts this table lacks (it
        must have been built with discount = alpha).  discount multiplies this model's own
        probabilities (1 for the main table)."""
        self.n_gram = int(n_gram)
        self.eps = float(np.float32(eps))
        self.discount = float(np.float32(discount))
        self.succ_ids = succ_ids
        self.succ_counts = succ_counts
        self.row_of = {tuple(int(t) for t in key): r for r, key in enumerate(keys)}
        self.miss = self._score(0.0)
        if backoff is not None:
            assert backoff.n_gram == self.n_gram - 1 and backoff.backoff is None
        self.backoff = backoff

    def _score(self, pr: float) -> np.float32:
        return min(np.float32(0.0), np.float32(math.log(self.discount * pr + self.eps)))

    def lookup(self, context) -> dict | None:
        """All successors of a context -> {token: s_ng}; None if the context is unseen (after
        the optional back-off to the context without its oldest token)."""
        context = tuple(int(t) for t in context)
        r = self.row_of.get(context)
        if r is None:
            return self.backoff.lookup(context[1:]) if self.backoff is not None else None
        counts = self.succ_counts[r]
        total = int(counts.astype(np.int64).sum())
        return {int(t): self._score(int(c) / total)
                for t, c in zip(self.succ_ids[r], counts) if c > 0}

    def score(self, row: dict | None, token: int) -> np.float32:
        if row is None:
            return self.miss
        return row.get(int(token), self.miss)
