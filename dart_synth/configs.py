"""Named workload shapes (Qwen3-family draft layers) used by tests and bench.

The five presets mirror the shapes the drafting step is evaluated on: a tiny
fp32 case the CPU oracle finishes in seconds, then bf16 drafts shaped like the
single decoder layer + LM head of Qwen3-1.7B / 8B / 14B / 32B (the draft layer's
head counts and widths are aligned with the target model, App. B "Training
Setup").  Pruning hyper-parameters default to the paper's beam width w = 20
(App. D); k and the node budget come from the preset.
"""
from __future__ import annotations

from dataclasses import dataclass, replace


@dataclass(frozen=True)
class DraftConfig:
    name: str
    d: int                # hidden size of the draft layer
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int              # SwiGLU intermediate size
    vocab: int
    ctx: int              # prefix length n (for batch > 1: the maximum)
    K: int                # draft length = number of logit rows
    topk: int             # per-position candidate count k
    n_gram: int           # N (2 = bigram, 3 = trigram)
    succ_per_key: int     # successors stored per N-gram context
    n_keys: int           # number of stored contexts
    budget: int           # tree node budget, root included (theta = budget-1)
    beam_w: int
    batch: int
    dtype: str            # "fp32" | "bf16": storage type of weights / hidden / KV
    qk_norm: bool
    rms_eps: float = 1e-6
    rope_base: float = 1e6
    ctx_min: int = 0      # batch > 1: ragged lengths drawn in [ctx_min, ctx]

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    def n_params(self) -> dict:
        attn = self.d * (2 * self.q_dim + 2 * self.kv_dim)
        mlp = 3 * self.d * self.ffn
        lm = self.d * self.vocab
        return {"attn": attn, "mlp": mlp, "lm_head": lm, "total": attn + mlp + lm}


CONFIGS = {
    "C1": DraftConfig("C1", d=512, n_q_heads=8, n_kv_heads=8, head_dim=64, ffn=1536,
                      vocab=8192, ctx=64, K=4, topk=4, n_gram=2, succ_per_key=16,
                      n_keys=8192, budget=16, beam_w=4, batch=1, dtype="fp32",
                      qk_norm=False),
    "C2": DraftConfig("C2", d=2048, n_q_heads=16, n_kv_heads=8, head_dim=128, ffn=6144,
                      vocab=151936, ctx=512, K=8, topk=8, n_gram=3, succ_per_key=64,
                      n_keys=1 << 20, budget=60, beam_w=20, batch=1, dtype="bf16",
                      qk_norm=True),
    "C3": DraftConfig("C3", d=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, ffn=12288,
                      vocab=151936, ctx=2048, K=8, topk=10, n_gram=3, succ_per_key=64,
                      n_keys=1 << 20, budget=60, beam_w=20, batch=1, dtype="bf16",
                      qk_norm=True),
    "C4": DraftConfig("C4", d=5120, n_q_heads=40, n_kv_heads=8, head_dim=128, ffn=17408,
                      vocab=151936, ctx=4096, K=8, topk=10, n_gram=3, succ_per_key=64,
                      n_keys=1 << 20, budget=60, beam_w=20, batch=1, dtype="bf16",
                      qk_norm=True),
    "C5": DraftConfig("C5", d=5120, n_q_heads=64, n_kv_heads=8, head_dim=128, ffn=25600,
                      vocab=151936, ctx=8192, K=8, topk=10, n_gram=3, succ_per_key=64,
                      n_keys=1 << 20, budget=60, beam_w=20, batch=16, dtype="bf16",
                      qk_norm=True, ctx_min=512),
}


def get_config(name: str) -> DraftConfig:
    return CONFIGS[name]


def scaled_config(base: str, **overrides) -> DraftConfig:
    """A preset with some fields replaced (small variants for parity tests)."""
    return replace(CONFIGS[base], **overrides)
