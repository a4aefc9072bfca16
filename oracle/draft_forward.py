"""Oracle: one forward pass of the DART draft layer (Sec. 3.2, Fig. 3).

Input sequence [z_1..z_n, MASK x (K-1)] -> a single pre-norm decoder layer
(RMSNorm, grouped-query attention with rotary positions, SwiGLU; "aligned with
the target model", App. B) under a strictly causal mask (Sec. 3.1) -> final norm
-> LM head.  K logit rows are read out: row 0 from the last prefix position, rows
1..K-1 from the mask positions ("shifted logits", Sec. 3.2).

`draft_forward` starts from the fused prefix representation z (width d);
`draft_forward_features` starts one step earlier, from the target model's raw outputs:
three concatenated hidden states through the FC layer, plus shifted token embeddings
(Sec. 3.2 "Draft model architecture").

Everything is fp64 numpy; stored bf16 / fp32 inputs are widened exactly first.
No blocking, caching or fusion: all T = n+K-1 rows go through K/V projection,
and attention is a per-query loop over the keys that query may see.
"""
from __future__ import annotations

import numpy as np


def widen(a: np.ndarray) -> np.ndarray:
    """Stored tensor -> fp64.  uint16 arrays hold bf16 bit patterns."""
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def rms_norm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """x / sqrt(mean(x^2) + eps) * gain over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def rope(x: np.ndarray, positions: np.ndarray, base: float) -> np.ndarray:
    """Rotary embedding on x[T][H][hd]; dimension i pairs with i + hd/2 and the
    pair rotates by angle position * base^(-2i/hd)."""
    hd = x.shape[-1]
    half = hd // 2
    inv_freq = base ** (-(2.0 * np.arange(half, dtype=np.float64)) / hd)
    ang = positions.astype(np.float64)[:, None] * inv_freq[None, :]
    cos, sin = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * cos - x2 * sin, x2 * cos + x1 * sin], axis=-1)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def attention_rows(q: np.ndarray, k: np.ndarray, v: np.ndarray, q_pos: np.ndarray) -> np.ndarray:
    """Causal grouped-query attention, one query at a time.

    q[R][Hq][hd] are the queries of absolute rows q_pos[R]; k, v[T][Hkv][hd] are the
    keys / values of rows 0..T-1.  The query of row r sees keys 0..r (the whole
    prefix plus the mask rows up to and including itself).
    """
    R, Hq, hd = q.shape
    Hkv = k.shape[1]
    group = Hq // Hkv
    out = np.zeros((R, Hq, hd), dtype=np.float64)
    for i in range(R):
        r = int(q_pos[i])
        for h in range(Hq):
            g = h // group
            s = k[: r + 1, g, :] @ q[i, h, :] / np.sqrt(float(hd))
            p = np.exp(s - s.max())
            p /= p.sum()
            out[i, h, :] = p @ v[: r + 1, g, :]
    return out


def draft_forward(cfg, weights: dict, hidden: np.ndarray, K: int,
                  return_intermediates: bool = False):
    """Logits [K][vocab] (fp64) for one prefix.

    cfg: object with d, n_q_heads, n_kv_heads, head_dim, ffn, vocab, qk_norm,
    rms_eps, rope_base.  weights: arrays named as in the draft layer
    ([out][in] matrices), stored fp32 or bf16 bits.  hidden: [n][d].
    """
    Hq, Hkv, hd = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    W = {name: widen(a) for name, a in weights.items() if name != "w_lm"}
    X = widen(hidden)
    n = X.shape[0]
    S = np.concatenate([X, W["mask_emb"][: K - 1]], axis=0)            # [T][d]
    T = n + K - 1
    rows = np.arange(n - 1, T)                                           # read-out rows

    a = rms_norm(S, W["w_in_norm"], cfg.rms_eps)
    k = (a @ W["wk"].T).reshape(T, Hkv, hd)
    v = (a @ W["wv"].T).reshape(T, Hkv, hd)
    q = (a[rows] @ W["wq"].T).reshape(K, Hq, hd)
    if cfg.qk_norm:
        q = rms_norm(q, W["q_norm"], cfg.rms_eps)
        k = rms_norm(k, W["k_norm"], cfg.rms_eps)
    q = rope(q, rows, cfg.rope_base)
    k = rope(k, np.arange(T), cfg.rope_base)

    o = attention_rows(q, k, v, rows).reshape(K, Hq * hd)
    y = S[rows] + o @ W["wo"].T
    b = rms_norm(y, W["w_post_norm"], cfg.rms_eps)
    u = y + (silu(b @ W["w_gate"].T) * (b @ W["w_up"].T)) @ W["w_down"].T
    f = rms_norm(u, W["w_final_norm"], cfg.rms_eps)

    logits = np.empty((K, cfg.vocab), dtype=np.float64)
    step = 8192
    for r0 in range(0, cfg.vocab, step):
        logits[:, r0:r0 + step] = f @ widen(weights["w_lm"][r0:r0 + step]).T
    if return_intermediates:
        return logits, {"a": a, "q": q, "k": k, "v": v, "o": o, "y": y, "b": b, "u": u, "f": f}
    return logits


def draft_forward_features(cfg, weights: dict, features: np.ndarray, next_tokens: np.ndarray,
                           K: int, return_intermediates: bool = False):
    """Logits [K][vocab] (fp64) from the target model's raw outputs (Sec. 3.2, Fig. 3, App. B).

    features [n][feat_dim]: the hidden states of three target layers, concatenated per
    position.  next_tokens [n]: the token that follows each prefix position (the last one is
    the freshly sampled t_{n+1}).  Steps, in the paper's order:
      g = FC(features)                         (output width d, App. B "Trainable parameters")
      e = Embedding(next_tokens)               (shifted token embeddings e_{2:n+1}, frozen table)
      z = [g ; e]                              (concatenated along the feature dimension)
      input sequence [z_1..z_n, MASK x (K-1)]  (a mask slot is a trainable 2d-wide row)
    The decoder layer takes the 2d-wide rows as attention input, each half under its own
    RMSNorm, and carries the g half as its residual stream; from the attention output on it
    is the layer of `draft_forward`.
    """
    Hq, Hkv, hd, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d
    W = {name: widen(a) for name, a in weights.items() if name not in ("w_lm", "embed")}
    F = widen(features)
    n = F.shape[0]
    g = F @ W["w_fc"].T                                                  # [n][d]
    e = widen(weights["embed"][np.asarray(next_tokens, dtype=np.int64)])  # [n][d]
    z = np.concatenate([g, e], axis=1)                                   # [n][2d]
    S = np.concatenate([z, W["mask_emb"][: K - 1]], axis=0)             # [T][2d]
    T = n + K - 1
    rows = np.arange(n - 1, T)

    a = np.concatenate([rms_norm(S[:, :d], W["w_in_norm"], cfg.rms_eps),
                        rms_norm(S[:, d:], W["w_emb_norm"], cfg.rms_eps)], axis=1)
    k = (a @ W["wk"].T).reshape(T, Hkv, hd)
    v = (a @ W["wv"].T).reshape(T, Hkv, hd)
    q = (a[rows] @ W["wq"].T).reshape(K, Hq, hd)
    if cfg.qk_norm:
        q = rms_norm(q, W["q_norm"], cfg.rms_eps)
        k = rms_norm(k, W["k_norm"], cfg.rms_eps)
    q = rope(q, rows, cfg.rope_base)
    k = rope(k, np.arange(T), cfg.rope_base)

    o = attention_rows(q, k, v, rows).reshape(K, Hq * hd)
    y = S[rows, :d] + o @ W["wo"].T
    b = rms_norm(y, W["w_post_norm"], cfg.rms_eps)
    u = y + (silu(b @ W["w_gate"].T) * (b @ W["w_up"].T)) @ W["w_down"].T
    f = rms_norm(u, W["w_final_norm"], cfg.rms_eps)

    logits = np.empty((K, cfg.vocab), dtype=np.float64)
    step = 8192
    for r0 in range(0, cfg.vocab, step):
        logits[:, r0:r0 + step] = f @ widen(weights["w_lm"][r0:r0 + step]).T
    if return_intermediates:
        return logits, {"g": g, "a": a, "o": o, "y": y, "u": u, "f": f}
    return logits


def lm_head_rows(weights: dict, f: np.ndarray, vocab_rows: np.ndarray) -> np.ndarray:
    """Logits of selected vocabulary rows only (sampled checks at full size)."""
    return f @ widen(weights["w_lm"][vocab_rows]).T
