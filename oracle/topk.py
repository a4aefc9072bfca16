"""Oracle: per-position candidate extraction (Alg. 1 "Top-k_i tokens from l_i" and
s_logit = log(softmax(l)_{i,t} + eps), App. D).

Top-k is the prefix of a full stable sort by (logit descending, token id
ascending).  The log-sum-exp and the score are evaluated in fp64 and the score is
rounded once to fp32, clamped to <= 0 (softmax + eps can exceed 1 by eps only).
"""
from __future__ import annotations

import numpy as np


def log_sum_exp(row: np.ndarray) -> float:
    row = row.astype(np.float64)
    m = row.max()
    return float(np.log(np.sum(np.exp(row - m))) + m)


def topk_rows(logits: np.ndarray, k: int, eps: float):
    """ids int32 [R][k], scores float32 [R][k] for logits [R][V]."""
    R, V = logits.shape
    ids = np.empty((R, k), dtype=np.int32)
    scores = np.empty((R, k), dtype=np.float32)
    eps64 = float(np.float32(eps))
    for r in range(R):
        row = logits[r].astype(np.float64)
        order = np.lexsort((np.arange(V), -row))          # full sort; ties -> lower id first
        top = order[:k]
        lse = log_sum_exp(row)
        s = np.log(np.exp(row[top] - lse) + eps64)
        ids[r] = top.astype(np.int32)
        scores[r] = np.minimum(np.float32(0.0), s.astype(np.float32))
    return ids, scores
