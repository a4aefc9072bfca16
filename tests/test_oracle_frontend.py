"""Pins for the oracle's front end (FC over concatenated target hidden states + shifted token
embeddings, Sec. 3.2): each reduces `draft_forward_features` to the already pinned
`draft_forward` or to a library routine, and planted mistakes must break them."""
import numpy as np
import torch

import dart_synth as ds
from oracle import draft_forward as odf

CFG = ds.scaled_config("C1", d=32, n_q_heads=4, n_kv_heads=2, head_dim=16, ffn=48, vocab=97, ctx=11,
                       K=4, qk_norm=True)


def _setup(seed=1, feat_dim=96):
    W = ds.make_frontend_weights(CFG, seed, feat_dim=feat_dim)
    feats, toks = ds.make_features(CFG, seed + 1, feat_dim=feat_dim)
    return W, feats, toks


def test_fc_is_a_plain_linear_layer():
    W, feats, toks = _setup()
    _, inter = odf.draft_forward_features(CFG, W, feats, toks, CFG.K, return_intermediates=True)
    ref = torch.nn.functional.linear(torch.from_numpy(feats.astype(np.float64)),
                                     torch.from_numpy(W["w_fc"].astype(np.float64))).numpy()
    np.testing.assert_allclose(inter["g"], ref, rtol=1e-12, atol=1e-12)


def test_g_half_alone_reduces_to_the_fused_input_path():
    """FC = [I 0 0] and Q/K/V blind to the embedding half: the layer sees exactly the prefix
    representation features[:, :d], so the result is draft_forward's on that input."""
    W, feats, toks = _setup()
    d = CFG.d
    W["w_fc"] = np.concatenate([np.eye(d, dtype=np.float32), np.zeros((d, 2 * d), np.float32)], axis=1)
    for name in ("wq", "wk", "wv"):
        W[name] = W[name].copy()
        W[name][:, d:] = 0
    got = odf.draft_forward_features(CFG, W, feats, toks, CFG.K)
    W0 = {k: v for k, v in W.items() if k not in ("w_fc", "embed", "w_emb_norm")}
    for name in ("wq", "wk", "wv"):
        W0[name] = W[name][:, :d].copy()
    W0["mask_emb"] = W["mask_emb"][:, :d].copy()
    ref = odf.draft_forward(CFG, W0, feats[:, :d].copy(), CFG.K)
    np.testing.assert_allclose(got, ref, rtol=1e-10, atol=1e-10)
    # planted mistake: halves swapped (z = [e ; g]) would make the layer blind to g instead
    Wsw = dict(W)
    for name in ("wq", "wk", "wv"):
        Wsw[name] = np.concatenate([W[name][:, d:], W[name][:, :d]], axis=1)
    assert np.abs(odf.draft_forward_features(CFG, Wsw, feats, toks, CFG.K) - ref).max() > 1e-3


def test_equal_halves_fold_into_summed_projections():
    """If the embedding of every row's NEXT token equals the row's g (and both halves share a
    gain and the mask halves are equal), then a = [h ; h] and W a = (W_g + W_e) h: the fused
    path with summed projection columns.  Uses the shifted index: row i reads next_tokens[i]."""
    W, feats, toks = _setup()
    d = CFG.d
    n = feats.shape[0]
    toks = np.random.default_rng(3).permutation(CFG.vocab)[:n].astype(np.int32)   # distinct tokens
    g = feats.astype(np.float64) @ W["w_fc"].astype(np.float64).T
    W["embed"] = W["embed"].astype(np.float64)
    W["embed"][toks] = g                                  # e_i = g_i exactly (fp64 table)
    W["w_emb_norm"] = W["w_in_norm"].copy()
    W["mask_emb"] = W["mask_emb"].copy()
    W["mask_emb"][:, d:] = W["mask_emb"][:, :d]
    got = odf.draft_forward_features(CFG, W, feats, toks, CFG.K)
    W0 = {k: v for k, v in W.items() if k not in ("w_fc", "embed", "w_emb_norm")}
    for name in ("wq", "wk", "wv"):
        W0[name] = (W[name][:, :d].astype(np.float64) + W[name][:, d:].astype(np.float64))
    W0["mask_emb"] = W["mask_emb"][:, :d].copy()
    ref = odf.draft_forward(CFG, W0, g, CFG.K)
    np.testing.assert_allclose(got, ref, rtol=1e-9, atol=1e-9)
    # planted mistake: unshifted embeddings (row i reading the token of row i-1) break it
    bad = odf.draft_forward_features(CFG, W, feats, np.roll(toks, 1), CFG.K)
    assert np.abs(bad - ref).max() > 1e-3
    # planted mistake: the embedding half normed with the wrong gain breaks it
    W2 = dict(W)
    W2["w_emb_norm"] = W["w_in_norm"] * 1.5
    assert np.abs(odf.draft_forward_features(CFG, W2, feats, toks, CFG.K) - ref).max() > 1e-3


def test_residual_is_the_g_half():
    """With Wo = 0 and Wdown = 0 the layer is the identity on its residual stream: logits =
    Wlm . RMSNorm(g of the read-out rows) -- a closed form that an e-half or 2d-wide residual
    would not satisfy."""
    W, feats, toks = _setup()
    d = CFG.d
    W["wo"] = np.zeros_like(W["wo"])
    W["w_down"] = np.zeros_like(W["w_down"])
    got = odf.draft_forward_features(CFG, W, feats, toks, CFG.K)
    g_last = feats[-1].astype(np.float64) @ W["w_fc"].astype(np.float64).T
    res = np.concatenate([g_last[None], W["mask_emb"][: CFG.K - 1, :d].astype(np.float64)], axis=0)
    f = odf.rms_norm(res, W["w_final_norm"].astype(np.float64), CFG.rms_eps)
    np.testing.assert_allclose(got, f @ W["w_lm"].astype(np.float64).T, rtol=1e-10, atol=1e-10)
