"""Seeded weights and hidden states, in the storage format the path reads.

Recipe: projection / LM-head weights ~ N(0, 0.02); RMSNorm gains ~ 1 + 0.1 N(0, 1)
(non-trivial so that a mis-applied gain shows up in parity); mask embeddings
~ N(0, 0.02); hidden states ~ N(0, 1).  For the bf16 presets every tensor is
drawn in fp32 and rounded once (round-to-nearest-even) to bf16; the returned
arrays hold the bf16 bit patterns as uint16, and both the oracle and the HIP
path read exactly those bits.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor

import numpy as np

from .configs import DraftConfig

# name -> (shape builder, kind); all matrices are [out_features][in_features] row-major.
WEIGHT_NAMES = (
    "w_in_norm", "wq", "wk", "wv", "q_norm", "k_norm", "wo", "w_post_norm",
    "w_gate", "w_up", "w_down", "w_final_norm", "w_lm", "mask_emb",
)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even), return the bits as uint16."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to fp32 exactly."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _shapes(cfg: DraftConfig, max_K: int) -> dict:
    return {
        "w_in_norm": (cfg.d,), "wq": (cfg.q_dim, cfg.d), "wk": (cfg.kv_dim, cfg.d),
        "wv": (cfg.kv_dim, cfg.d), "q_norm": (cfg.head_dim,), "k_norm": (cfg.head_dim,),
        "wo": (cfg.d, cfg.q_dim), "w_post_norm": (cfg.d,),
        "w_gate": (cfg.ffn, cfg.d), "w_up": (cfg.ffn, cfg.d), "w_down": (cfg.d, cfg.ffn),
        "w_final_norm": (cfg.d,), "w_lm": (cfg.vocab, cfg.d),
        "mask_emb": (max(max_K - 1, 1), cfg.d),
    }


def _draw(seed_words, shape, kind: str, store_bf16: bool) -> np.ndarray:
    """Draw one tensor in row chunks, each chunk from its own seeded stream (so chunks can be
    drawn in parallel and the result does not depend on the number of workers)."""
    shape = tuple(shape)
    rows = shape[0]
    cols = int(np.prod(shape[1:])) if len(shape) > 1 else 1
    out = np.empty(shape, dtype=np.uint16 if store_bf16 else np.float32)
    flat = out.reshape(rows, cols)
    step = max(1, (1 << 24) // cols)

    def fill(c: int) -> None:
        r0, r1 = c * step, min(rows, (c + 1) * step)
        rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([*seed_words, c])))
        z = rng.standard_normal((r1 - r0, cols), dtype=np.float32)
        if kind == "gain":
            z = np.float32(1.0) + np.float32(0.1) * z
        elif kind == "small":
            z = np.float32(0.02) * z
        flat[r0:r1] = f32_to_bf16_bits(z) if store_bf16 else z

    n_chunks = (rows + step - 1) // step
    if n_chunks == 1:
        fill(0)
    else:
        with ThreadPoolExecutor(max_workers=8) as pool:
            list(pool.map(fill, range(n_chunks)))
    return out


def make_weights(cfg: DraftConfig, seed: int, max_K: int | None = None) -> dict:
    """All draft-layer tensors for one preset; uint16 (bf16 bits) or float32 arrays."""
    max_K = cfg.K if max_K is None else max_K
    store_bf16 = cfg.dtype == "bf16"
    out = {}
    for idx, (name, shape) in enumerate(_shapes(cfg, max_K).items()):
        kind = "gain" if name in ("w_in_norm", "q_norm", "k_norm", "w_post_norm",
                                  "w_final_norm") else "small"
        out[name] = _draw([seed, 101, idx], shape, kind, store_bf16)
    return out


def make_frontend_weights(cfg: DraftConfig, seed: int, max_K: int | None = None,
                          feat_dim: int | None = None) -> dict:
    """Draft-layer tensors for the variant that starts from the target's raw outputs: the
    FC layer w_fc [d][feat_dim] (feat_dim = 3 d: three target layers), the frozen embedding
    table embed [vocab][d], a second input gain w_emb_norm [d], Q/K/V over the 2d-wide input
    and 2d-wide mask rows.  The remaining tensors are those of make_weights (same seed, same
    values)."""
    max_K = cfg.K if max_K is None else max_K
    feat_dim = 3 * cfg.d if feat_dim is None else feat_dim
    store_bf16 = cfg.dtype == "bf16"
    out = make_weights(cfg, seed, max_K)
    extra = {"wq": ((cfg.q_dim, 2 * cfg.d), "small"), "wk": ((cfg.kv_dim, 2 * cfg.d), "small"),
             "wv": ((cfg.kv_dim, 2 * cfg.d), "small"),
             "mask_emb": ((max(max_K - 1, 1), 2 * cfg.d), "small"),
             "w_fc": ((cfg.d, feat_dim), "fc"), "embed": ((cfg.vocab, cfg.d), "unit"),
             "w_emb_norm": ((cfg.d,), "gain")}
    for idx, (name, (shape, kind)) in enumerate(extra.items()):
        t = _draw([seed, 404, idx], shape, "unit" if kind == "fc" else kind, False)
        if kind == "fc":                       # N(0, 1/feat_dim): g rows of unit scale
            t = t * np.float32(1.0 / np.sqrt(feat_dim))
        out[name] = f32_to_bf16_bits(t) if store_bf16 else t
    return out


def make_features(cfg: DraftConfig, seed: int, n: int | None = None, feat_dim: int | None = None):
    """Raw target outputs of an n-token prefix: features [n][feat_dim] ~ N(0, 1) (three
    concatenated hidden states) and next_tokens [n] int32, uniform over the vocabulary (the
    token following each position; the last one stands for the sampled t_{n+1})."""
    n = cfg.ctx if n is None else n
    feat_dim = 3 * cfg.d if feat_dim is None else feat_dim
    feats = _draw([seed, 505], (n, feat_dim), "unit", cfg.dtype == "bf16")
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 506])))
    return feats, rng.integers(0, cfg.vocab, size=n).astype(np.int32)


def make_hidden(cfg: DraftConfig, seed: int, n: int | None = None) -> np.ndarray:
    """Target hidden states of an n-token prefix, N(0, 1), [n][d]."""
    n = cfg.ctx if n is None else n
    return _draw([seed, 202], (n, cfg.d), "unit", cfg.dtype == "bf16")


def make_ragged_lengths(cfg: DraftConfig, seed: int) -> np.ndarray:
    """Batch of context lengths, uniform on [ctx_min, ctx] (ragged batched preset)."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 303])))
    lo = cfg.ctx_min if cfg.ctx_min > 0 else cfg.ctx
    return rng.integers(lo, cfg.ctx + 1, size=cfg.batch).astype(np.int32)
