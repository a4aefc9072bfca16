"""Pins for the oracle's draft forward (Sec. 3.1, 3.2, App. B): each piece is checked
against a library routine or a closed form, and the whole layer against an
installed-library Qwen3 / LLaMA decoder layer used as a black box."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import dart_synth as ds
from oracle import draft_forward as odf

TINY = ds.scaled_config("C1", d=64, n_q_heads=4, n_kv_heads=2, head_dim=16, ffn=96,
                        vocab=100, ctx=9, K=4)


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def test_rms_norm_matches_library():
    x, g = _rand((5, 32), 0), _rand((32,), 1)
    ref = F.rms_norm(torch.from_numpy(x), (32,), torch.from_numpy(g), eps=1e-6).numpy()
    np.testing.assert_allclose(odf.rms_norm(x, g, 1e-6), ref, rtol=1e-12, atol=1e-12)


def test_rms_norm_eps_matters():
    x = np.full((1, 4), 1e-3)
    out = odf.rms_norm(x, np.ones(4), 1e-6)
    np.testing.assert_allclose(out, 1e-3 / np.sqrt(1e-6 + 1e-6), rtol=1e-12)


def test_silu_matches_library():
    x = _rand((7, 9), 2) * 4
    np.testing.assert_allclose(odf.silu(x), F.silu(torch.from_numpy(x)).numpy(), rtol=1e-12,
                               atol=1e-12)


def test_rope_is_a_complex_rotation_of_half_split_pairs():
    T, H, hd, base = 6, 2, 8, 1e4
    x = _rand((T, H, hd), 3)
    pos = np.array([0, 1, 2, 5, 9, 100])
    out = odf.rope(x, pos, base)
    half = hd // 2
    z = x[..., :half] + 1j * x[..., half:]
    theta = pos[:, None] * base ** (-2.0 * np.arange(half) / hd)
    zr = z * np.exp(1j * theta)[:, None, :]
    np.testing.assert_allclose(out[..., :half], zr.real, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(out[..., half:], zr.imag, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(out[0], x[0])          # position 0 is the identity


def test_attention_matches_library_sdpa_with_explicit_mask():
    T, R, Hq, Hkv, hd = 11, 4, 6, 2, 8
    q, k, v = _rand((R, Hq, hd), 4), _rand((T, Hkv, hd), 5), _rand((T, Hkv, hd), 6)
    rows = np.arange(T - R, T)
    out = odf.attention_rows(q, k, v, rows)
    allowed = torch.from_numpy(np.arange(T)[None, :] <= rows[:, None])          # [R][T]
    kk = torch.from_numpy(k).repeat_interleave(Hq // Hkv, dim=1).permute(1, 0, 2)
    vv = torch.from_numpy(v).repeat_interleave(Hq // Hkv, dim=1).permute(1, 0, 2)
    ref = F.scaled_dot_product_attention(torch.from_numpy(q).permute(1, 0, 2)[None], kk[None],
                                         vv[None], attn_mask=allowed[None, None])
    np.testing.assert_allclose(out, ref[0].permute(1, 0, 2).numpy(), rtol=1e-10, atol=1e-12)


def test_attention_single_key_returns_value_and_uniform_keys_average():
    q, k, v = _rand((1, 2, 4), 7), _rand((1, 2, 4), 8), _rand((1, 2, 4), 9)
    np.testing.assert_allclose(odf.attention_rows(q, k, v, np.array([0])), v)
    k5 = np.repeat(k, 5, axis=0)
    v5 = _rand((5, 2, 4), 10)
    out = odf.attention_rows(q, k5, v5, np.array([4]))
    np.testing.assert_allclose(out[0], v5.mean(axis=0), rtol=1e-12)


def _library_logits(cfg, W, hidden, K):
    """The same layer assembled from an installed transformer library (black box)."""
    import transformers
    common = dict(vocab_size=cfg.vocab, hidden_size=cfg.d, intermediate_size=cfg.ffn,
                  num_hidden_layers=1, num_attention_heads=cfg.n_q_heads,
                  num_key_value_heads=cfg.n_kv_heads, head_dim=cfg.head_dim,
                  rms_norm_eps=cfg.rms_eps, rope_theta=cfg.rope_base,
                  tie_word_embeddings=False, attention_bias=False,
                  max_position_embeddings=4096)
    if cfg.qk_norm:
        model = transformers.Qwen3ForCausalLM(transformers.Qwen3Config(**common))
    else:
        model = transformers.LlamaForCausalLM(transformers.LlamaConfig(mlp_bias=False, **common))
    model = model.double().eval()
    names = {"model.layers.0.self_attn.q_proj.weight": "wq",
             "model.layers.0.self_attn.k_proj.weight": "wk",
             "model.layers.0.self_attn.v_proj.weight": "wv",
             "model.layers.0.self_attn.o_proj.weight": "wo",
             "model.layers.0.mlp.gate_proj.weight": "w_gate",
             "model.layers.0.mlp.up_proj.weight": "w_up",
             "model.layers.0.mlp.down_proj.weight": "w_down",
             "model.layers.0.input_layernorm.weight": "w_in_norm",
             "model.layers.0.post_attention_layernorm.weight": "w_post_norm",
             "model.norm.weight": "w_final_norm", "lm_head.weight": "w_lm"}
    if cfg.qk_norm:
        names["model.layers.0.self_attn.q_norm.weight"] = "q_norm"
        names["model.layers.0.self_attn.k_norm.weight"] = "k_norm"
    sd = model.state_dict()
    for lib_name, ours in names.items():
        assert tuple(sd[lib_name].shape) == W[ours].shape, lib_name
        sd[lib_name].copy_(torch.from_numpy(odf.widen(W[ours])))
    S = np.concatenate([odf.widen(hidden), odf.widen(W["mask_emb"])[: K - 1]], axis=0)
    with torch.no_grad():
        out = model(inputs_embeds=torch.from_numpy(S)[None]).logits[0].numpy()
    n = hidden.shape[0]
    return out[n - 1: n + K - 1]


@pytest.mark.parametrize("qk_norm", [True, False])
def test_whole_layer_matches_library_decoder(qk_norm):
    cfg = ds.scaled_config("C1", d=64, n_q_heads=4, n_kv_heads=2, head_dim=16, ffn=96,
                           vocab=100, ctx=9, K=4, qk_norm=qk_norm)
    W = ds.make_weights(cfg, seed=11)
    W = {name: (a * 5 if name.startswith("w") and a.ndim == 2 else a) for name, a in W.items()}
    hidden = ds.make_hidden(cfg, seed=12)
    ours = odf.draft_forward(cfg, W, hidden, cfg.K)
    ref = _library_logits(cfg, W, hidden, cfg.K)
    assert np.abs(ref).max() > 1e-2
    # the library evaluates its rotary angles in fp32 even in a double model, hence 1e-5
    np.testing.assert_allclose(ours, ref, rtol=1e-4, atol=1e-5)


def test_bf16_storage_is_widened_exactly():
    cfg = ds.scaled_config("C1", d=64, n_q_heads=4, n_kv_heads=2, head_dim=16, ffn=96,
                           vocab=100, ctx=9, K=3, dtype="bf16", qk_norm=True)
    W = ds.make_weights(cfg, seed=13)
    hidden = ds.make_hidden(cfg, seed=14)
    assert W["wq"].dtype == np.uint16
    Wf = {name: ds.bf16_bits_to_f32(a) for name, a in W.items()}
    a = odf.draft_forward(cfg, W, hidden, cfg.K)
    b = odf.draft_forward(cfg, Wf, ds.bf16_bits_to_f32(hidden), cfg.K)
    np.testing.assert_array_equal(a, b)
    np.testing.assert_array_equal(
        odf.widen(np.array([0x3F80, 0xC000, 0x3DCD], dtype=np.uint16)),
        np.array([1.0, -2.0, 0.10009765625]))


def test_closed_form_when_attention_and_mlp_outputs_are_zero():
    cfg = TINY
    W = ds.make_weights(cfg, seed=15)
    W["wo"] = np.zeros_like(W["wo"])
    W["w_down"] = np.zeros_like(W["w_down"])
    hidden = ds.make_hidden(cfg, seed=16)
    out = odf.draft_forward(cfg, W, hidden, cfg.K)
    S = np.concatenate([hidden, W["mask_emb"][: cfg.K - 1]]).astype(np.float64)
    rows = S[cfg.ctx - 1:]
    f = rows / np.sqrt((rows ** 2).mean(-1, keepdims=True) + cfg.rms_eps) * W["w_final_norm"]
    np.testing.assert_allclose(out, f @ W["w_lm"].astype(np.float64).T, rtol=1e-12)


def test_row_readout_and_causality():
    cfg = TINY
    K, n = cfg.K, cfg.ctx
    W = ds.make_weights(cfg, seed=17)
    W = {name: (a * 5 if a.ndim == 2 and name != "mask_emb" else a) for name, a in W.items()}
    hidden = ds.make_hidden(cfg, seed=18)
    base = odf.draft_forward(cfg, W, hidden, K)
    # mask slot s feeds output row s; perturbing it may change only rows >= s
    for s in range(1, K):
        W2 = dict(W)
        W2["mask_emb"] = W["mask_emb"].copy()
        W2["mask_emb"][s - 1] += 1.0
        out = odf.draft_forward(cfg, W2, hidden, K)
        changed = np.abs(out - base).max(axis=1) > 1e-9
        assert not changed[:s].any() and changed[s:].all(), (s, changed)
    # any prefix row (the first, a middle one, the last) reaches all K rows
    for r in (0, n // 2, n - 1):
        h2 = hidden.copy()
        h2[r] += 1.0
        out = odf.draft_forward(cfg, W, h2, K)
        assert (np.abs(out - base).max(axis=1) > 1e-9).all()
    # a shorter draft is a prefix of a longer one (rows do not depend on later masks)
    np.testing.assert_allclose(odf.draft_forward(cfg, W, hidden, 2), base[:2], rtol=1e-12)


def test_gqa_equals_mha_with_duplicated_kv_heads():
    cfg = TINY
    W = ds.make_weights(cfg, seed=19)
    hidden = ds.make_hidden(cfg, seed=20)
    g = cfg.n_q_heads // cfg.n_kv_heads
    mha = ds.scaled_config("C1", d=64, n_q_heads=4, n_kv_heads=4, head_dim=16, ffn=96,
                           vocab=100, ctx=9, K=4)
    W2 = dict(W)
    for name in ("wk", "wv"):
        w = W[name].reshape(cfg.n_kv_heads, cfg.head_dim, cfg.d)
        W2[name] = np.repeat(w, g, axis=0).reshape(-1, cfg.d)
    np.testing.assert_allclose(odf.draft_forward(mha, W2, hidden, 4),
                               odf.draft_forward(cfg, W, hidden, 4), rtol=1e-10, atol=1e-13)


def test_single_hot_final_state_reads_a_column_of_the_lm_head():
    W = ds.make_weights(TINY, seed=21)
    f = np.zeros((1, TINY.d))
    f[0, 5] = 2.0
    rows = np.array([3, 50, 99])
    np.testing.assert_allclose(odf.lm_head_rows(W, f, rows)[0],
                               2.0 * W["w_lm"][rows, 5].astype(np.float64))


# ---- planted mistakes: each plausible slip must break the library pin -------------------

def _wrong_rope_interleaved(x, positions, base):
    hd = x.shape[-1]
    inv = base ** (-(2.0 * np.arange(hd // 2)) / hd)
    ang = positions.astype(np.float64)[:, None] * inv[None, :]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    out = np.empty_like(x)
    out[..., 0::2] = x[..., 0::2] * c - x[..., 1::2] * s
    out[..., 1::2] = x[..., 1::2] * c + x[..., 0::2] * s
    return out


_ATTENTION = odf.attention_rows


def _wrong_attention_excludes_self(q, k, v, q_pos):
    return _ATTENTION(q, k, v, q_pos - 1)


def _wrong_attention_head_mapping(q, k, v, q_pos):
    Hq, Hkv = q.shape[1], k.shape[1]
    perm = [(h % Hkv) * (Hq // Hkv) + h // Hkv for h in range(Hq)]
    return _ATTENTION(q[:, perm], k, v, q_pos)


@pytest.mark.parametrize("name,wrong", [
    ("rope", _wrong_rope_interleaved),
    ("attention_rows", _wrong_attention_excludes_self),
    ("attention_rows", _wrong_attention_head_mapping),
    ("silu", lambda x: x / (1.0 + np.exp(x))),
    ("rms_norm", lambda x, g, eps: x / np.sqrt(np.mean(x * x, -1, keepdims=True)) * g * 1.01),
])
def test_planted_mistake_is_caught_by_library_pin(monkeypatch, name, wrong):
    monkeypatch.setattr(odf, name, wrong)
    with pytest.raises(AssertionError):
        test_whole_layer_matches_library_decoder(True)
