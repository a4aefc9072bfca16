"""Seeded N-gram count tables and prune-only workloads.

Stands in for the paper's 3-gram trie built from a text corpus (App. C): that
corpus is not available, so contexts and successors are drawn from a bounded
power law (exponent 1.1, "Zipf(1.1)") over a seeded permutation of the token
ids.  Only raw *counts* are produced here; turning counts into probabilities and
log-scores is the method's arithmetic and is done separately by the oracle and
by the library.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from .configs import DraftConfig

ZIPF_A = 1.1
COUNT_SCALE = 1000.0


@dataclass
class NgramCounts:
    n_gram: int               # N; a context is the previous N-1 tokens
    keys: np.ndarray          # int32 [n_keys][N-1], oldest token first, all rows distinct
    succ_ids: np.ndarray      # int32 [n_keys][S], distinct within a row, -1 = unused slot
    succ_counts: np.ndarray   # int32 [n_keys][S], > 0 where used, 0 where unused


@dataclass
class PruneCase:
    ids: np.ndarray           # int32 [K][k] candidate token ids per level, best first
    scores: np.ndarray        # float32 [K][k] candidate log-scores (<= 0), descending
    ctx_tail: np.ndarray      # int32 [N-1] last real tokens, root (t_{n+1}) last
    table: NgramCounts


def _zipf_ranks(rng: np.random.Generator, size, vocab: int) -> np.ndarray:
    """Ranks in [0, vocab) from the continuous power law x^-a on [1, vocab+1)."""
    u = rng.random(size)
    e = 1.0 - ZIPF_A
    x = (1.0 + u * ((vocab + 1.0) ** e - 1.0)) ** (1.0 / e)
    return np.minimum(np.floor(x).astype(np.int64) - 1, vocab - 1)


def _distinct_rows(ranks: np.ndarray, vocab: int) -> np.ndarray:
    """Make every row's ranks distinct: sort, then push collisions to the next free rank."""
    r = np.sort(ranks, axis=1)
    j = np.arange(r.shape[1], dtype=np.int64)[None, :]
    r = np.maximum.accumulate(r - j, axis=1) + j
    over = r[:, -1:] - (vocab - 1)
    return r - np.maximum(over, 0)


def _counts_row(S: int) -> np.ndarray:
    j = np.arange(S, dtype=np.float64)
    return np.ceil(COUNT_SCALE * (j + 1.0) ** (-ZIPF_A)).astype(np.int32)


def make_ngram_counts(cfg: DraftConfig, seed: int, n_keys: int | None = None) -> NgramCounts:
    """Count table of a preset: `n_keys` contexts with `succ_per_key` successors each.

    Successor j of a row (ascending Zipf rank) carries count ceil(1000 (j+1)^-1.1).
    The bigram preset whose n_keys equals the vocabulary is dense: every token is
    a context.
    """
    n_keys = cfg.n_keys if n_keys is None else n_keys
    S, V, ctx_len = cfg.succ_per_key, cfg.vocab, cfg.n_gram - 1
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 404])))
    perm = rng.permutation(V).astype(np.int32)

    if ctx_len == 1 and n_keys == V:
        keys = np.arange(V, dtype=np.int32)[:, None]
    else:
        packed = np.empty(0, dtype=np.int64)
        while packed.size < n_keys:
            draw = _zipf_ranks(rng, (int(n_keys * 1.5) + 16, ctx_len), V)
            p = np.zeros(draw.shape[0], dtype=np.int64)
            for c in range(ctx_len):
                p = p * V + draw[:, c]
            both = np.concatenate([packed, p])
            _, first = np.unique(both, return_index=True)
            packed = both[np.sort(first)]
        packed = packed[:n_keys]
        keys = np.empty((n_keys, ctx_len), dtype=np.int32)
        for c in range(ctx_len - 1, -1, -1):
            keys[:, c] = perm[packed % V]
            packed = packed // V

    succ_ids = np.empty((n_keys, S), dtype=np.int32)
    step = 1 << 16
    for r0 in range(0, n_keys, step):
        r1 = min(n_keys, r0 + step)
        ranks = _distinct_rows(_zipf_ranks(rng, (r1 - r0, S), V), V)
        succ_ids[r0:r1] = perm[ranks]
    succ_counts = np.broadcast_to(_counts_row(S), (n_keys, S)).copy()
    return NgramCounts(cfg.n_gram, keys, succ_ids, succ_counts)


def make_prune_case(seed: int, *, vocab: int, K: int, k: int, n_gram: int, S: int,
                    n_filler_keys: int = 256, p_key: float = 0.5,
                    p_succ: float = 0.5) -> PruneCase:
    """Prune-only workload with hits, partial hits and misses planted on purpose.

    Candidate ids per level are distinct Zipf draws; scores are descending
    negative log-like values.  For about `p_key` of the contexts a beam entry can
    present at each level, a table row is planted that contains about `p_succ` of
    that level's candidates, the rest of the row being Zipf filler (some rows are
    left partly unused).  `n_filler_keys` unrelated rows are added on top.
    """
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 505])))
    ctx_len = n_gram - 1
    perm = rng.permutation(vocab).astype(np.int32)
    ids = perm[_distinct_rows(_zipf_ranks(rng, (K, k), vocab), vocab)]
    for L in range(K):
        rng.shuffle(ids[L])
    gaps = rng.exponential(0.7, size=(K, k)) + 1e-3
    scores = (-np.cumsum(gaps, axis=1)).astype(np.float32)
    ctx_tail = perm[_zipf_ranks(rng, ctx_len, vocab)].astype(np.int32)
    root = int(ctx_tail[-1])

    assert n_gram in (2, 3)
    contexts = {}          # tuple -> level whose candidates the row should contain
    for L in range(K):
        if L == 0:
            cand_ctx = [tuple(int(t) for t in ctx_tail)]
        elif ctx_len == 1:
            cand_ctx = [(int(b),) for b in ids[L - 1]]
        else:
            prev2 = [root] if L == 1 else [int(a) for a in ids[L - 2]]
            cand_ctx = [(a, int(b)) for a in prev2 for b in ids[L - 1]]
        for c in cand_ctx:
            if c not in contexts and rng.random() < p_key:
                contexts[c] = L
    n_fill = n_filler_keys
    while n_fill > 0:
        c = tuple(int(t) for t in perm[_zipf_ranks(rng, ctx_len, vocab)])
        if c not in contexts:
            contexts[c] = -1
            n_fill -= 1

    n_keys = len(contexts)
    keys = np.empty((n_keys, ctx_len), dtype=np.int32)
    succ_ids = np.full((n_keys, S), -1, dtype=np.int32)
    succ_counts = np.zeros((n_keys, S), dtype=np.int32)
    base_counts = _counts_row(S)
    order = rng.permutation(n_keys)
    for row, (c, L) in zip(order, contexts.items()):
        keys[row] = c
        used = int(rng.integers(1, S + 1)) if rng.random() < 0.3 else S
        chosen = []
        if L >= 0:
            chosen = [int(t) for t in ids[L] if rng.random() < p_succ][:used]
        have = set(chosen)
        while len(chosen) < used:
            t = int(perm[_zipf_ranks(rng, (), vocab)])
            if t not in have:
                have.add(t)
                chosen.append(t)
        chosen = np.array(chosen, dtype=np.int32)
        rng.shuffle(chosen)
        succ_ids[row, :used] = chosen
        succ_counts[row, :used] = base_counts[:used]
    return PruneCase(ids.astype(np.int32), scores, ctx_tail,
                     NgramCounts(n_gram, keys, succ_ids, succ_counts))


def make_bulk_trigram_counts(n_keys: int, S: int, vocab: int, seed: int) -> NgramCounts:
    """A trigram count table of `n_keys` contexts built arithmetically, for tables far larger
    than the presets' (2^24 contexts and more) where rejection sampling of Zipf contexts and a
    Python-side index would take minutes.

    Context r is the pair (p // vocab, p % vocab) of p = (r * mult + off) mod vocab^2 with mult
    coprime to vocab^2, so all contexts are distinct and `bulk_row_of` finds the row of a
    context without an index.  Successor j of row r is (a_r + j * s_r) mod vocab with s_r coprime
    to vocab (distinct within the row); counts follow ceil(1000 (j+1)^-1.1) as in the presets.
    """
    import math
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 606])))
    V2 = vocab * vocab
    assert n_keys <= V2 and V2 < (1 << 36) and n_keys <= (1 << 26)
    mult, off = _bulk_params(vocab, seed)
    strides = np.array([s for s in range(3, 4 * vocab // 5, 2) if math.gcd(s, vocab) == 1][:4096],
                       dtype=np.int64)
    keys = np.empty((n_keys, 2), dtype=np.int32)
    succ_ids = np.empty((n_keys, S), dtype=np.int32)
    j = np.arange(S, dtype=np.int32)[None, :]      # j * s_r < 64 * vocab: int32 arithmetic suffices
    step = 1 << 20
    for r0 in range(0, n_keys, step):
        r = np.arange(r0, min(n_keys, r0 + step), dtype=np.int64)
        p = (r * mult + off) % V2
        keys[r0:r0 + r.size, 0] = p // vocab
        keys[r0:r0 + r.size, 1] = p % vocab
        a = ((r * 2654435761 + seed) % vocab).astype(np.int32)
        s = strides[(r * 40503 + 17) % strides.size].astype(np.int32)
        block = succ_ids[r0:r0 + r.size]
        np.multiply(j, s[:, None], out=block)
        block += a[:, None]
        block %= np.int32(vocab)
    succ_counts = np.broadcast_to(_counts_row(S), (n_keys, S)).copy()
    del rng
    return NgramCounts(3, keys, succ_ids, succ_counts)


def _bulk_params(vocab: int, seed: int):
    import math
    V2 = vocab * vocab
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 607])))
    while True:
        mult = int(rng.integers(1 << 20, 1 << 34))
        if math.gcd(mult, V2) == 1:
            break
    return mult, int(rng.integers(0, V2))


def bulk_row_of(n_keys: int, vocab: int, seed: int, prev: int, tok: int) -> int:
    """Row of context (prev, tok) in make_bulk_trigram_counts(n_keys, ., vocab, seed), or -1."""
    V2 = vocab * vocab
    mult, off = _bulk_params(vocab, seed)
    r = ((prev * vocab + tok - off) * pow(mult, -1, V2)) % V2
    return int(r) if r < n_keys else -1


def plant_prune_case(table: NgramCounts, n_keys: int, vocab: int, table_seed: int, seed: int, *,
                     K: int, k: int, p_key: float = 0.5, p_succ: float = 0.5) -> PruneCase:
    """A prune-only case whose contexts really hit a bulk table: candidate lists are drawn, and
    for about `p_key` of the contexts a beam entry can present (tail; (root, level-0 candidate);
    (candidate of level L-2, candidate of level L-1)) a row of the table is rewritten IN PLACE to
    that context with about `p_succ` of the next level's candidates among its successors.  A
    context that the bulk table already holds keeps its row (found with bulk_row_of).  Returns the
    case; `table` is modified."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 608])))
    S = table.succ_ids.shape[1]
    ids = np.stack([rng.choice(vocab, size=k, replace=False) for _ in range(K)]).astype(np.int32)
    gaps = rng.exponential(0.7, size=(K, k)) + 1e-3
    scores = (-np.cumsum(gaps, axis=1)).astype(np.float32)
    ctx_tail = rng.integers(0, vocab, size=2).astype(np.int32)
    root = int(ctx_tail[1])
    used_rows, planted = set(), set()
    for L in range(K):
        if L == 0:
            ctxs = [(int(ctx_tail[0]), root)]
        elif L == 1:
            ctxs = [(root, int(b)) for b in ids[0]]
        else:
            ctxs = [(int(a), int(b)) for a in ids[L - 2] for b in ids[L - 1]]
        for c in ctxs:
            if c in planted or rng.random() >= p_key:
                continue
            planted.add(c)
            row = bulk_row_of(n_keys, vocab, table_seed, *c)
            if row < 0:                       # not a bulk context: take over a row not yet used
                row = int(rng.integers(0, n_keys))
                while row in used_rows:
                    row = int(rng.integers(0, n_keys))
                # the row's old context disappears, the new one must not exist elsewhere: it does
                # not, since bulk_row_of found none and planted contexts are distinct
                table.keys[row] = c
            if row in used_rows:
                continue
            used_rows.add(row)
            chosen = [int(t) for t in ids[L] if rng.random() < p_succ]
            have = set(chosen)
            for t in table.succ_ids[row]:
                if len(chosen) == S:
                    break
                if int(t) not in have:
                    have.add(int(t))
                    chosen.append(int(t))
            chosen = np.array(chosen[:S], dtype=np.int32)
            rng.shuffle(chosen)
            table.succ_ids[row] = chosen
    return PruneCase(ids, scores, ctx_tail, table)


def make_backoff_counts(case: PruneCase, seed: int, *, vocab: int, S: int, p_key: float = 0.6,
                        p_succ: float = 0.5, n_filler_keys: int = 64) -> NgramCounts:
    """A bigram count table to go with a trigram prune case as its back-off: for about `p_key` of
    the tokens that can be the newest token of a context (the root and the candidates of every
    level but the last) a row is planted holding about `p_succ` of the next level's candidates
    plus filler; `n_filler_keys` unrelated rows are added.  Same row format as the main table."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 707])))
    K, k = case.ids.shape
    rows = {}                                   # newest token -> level whose candidates follow it
    rows_for = [(int(case.ctx_tail[-1]), 0)] + [(int(t), L + 1) for L in range(K - 1) for t in case.ids[L]]
    for tok, L in rows_for:
        if tok not in rows and rng.random() < p_key:
            rows[tok] = L
    while n_filler_keys > 0:
        tok = int(rng.integers(0, vocab))
        if tok not in rows:
            rows[tok] = -1
            n_filler_keys -= 1
    n = len(rows)
    keys = np.empty((n, 1), dtype=np.int32)
    succ_ids = np.full((n, S), -1, dtype=np.int32)
    succ_counts = np.zeros((n, S), dtype=np.int32)
    base = _counts_row(S)
    for r, (tok, L) in zip(rng.permutation(n), rows.items()):
        keys[r, 0] = tok
        used = int(rng.integers(1, S + 1)) if rng.random() < 0.3 else S
        chosen = [int(t) for t in case.ids[L] if rng.random() < p_succ][:used] if L >= 0 else []
        have = set(chosen)
        while len(chosen) < used:
            t = int(rng.integers(0, vocab))
            if t not in have:
                have.add(t)
                chosen.append(t)
        chosen = np.array(chosen, dtype=np.int32)
        rng.shuffle(chosen)
        succ_ids[r, :used] = chosen
        succ_counts[r, :used] = base[:used]
    return NgramCounts(2, keys, succ_ids, succ_counts)
