"""GPU parity: dart_draft_forward (HIP, through the C ABI) against the CPU oracle."""
import numpy as np
import pytest

import dart_synth as ds
from oracle import draft_forward as odf
from util_gpu import hidden_to_device, logits_close, make_context

pytestmark = pytest.mark.gpu

# fp32 path: fp32 accumulation of <= 1536-term dot products of O(1) values -> ~1e-6 relative.
F32_TOL = dict(atol=2e-4, rtol=2e-4)
# bf16 path: tolerance stated for the build: max-abs 2e-2 / relative 1e-2 against the oracle.
BF16_TOL = dict(atol=2e-2, rtol=1e-2)

SMALL_BF16 = {
    # ragged everything: vocab not a multiple of 16, ctx not a multiple of 32, hd 64, K 5
    "tiny64": ds.scaled_config("C2", d=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=512,
                               vocab=1000, ctx=70, K=5),
    # hd 128, 4 query heads per K/V head, several key splits, ragged tail
    "mid128": ds.scaled_config("C2", d=512, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn=1536,
                               vocab=8192, ctx=301, K=8),
    # ffn long enough that the down projection is cut into k-chunks; 5 heads per K/V head; K 16
    "chunked": ds.scaled_config("C2", d=256, n_q_heads=5, n_kv_heads=1, head_dim=128, ffn=5632,
                                vocab=2048, ctx=130, K=16),
    # d beyond one k-chunk of the skinny kernel: the LM head goes through chunk partials
    "long_d": ds.scaled_config("C2", d=8192, n_q_heads=4, n_kv_heads=2, head_dim=128, ffn=1024,
                               vocab=3000, ctx=100, K=8),
    "long_d_16rows": ds.scaled_config("C2", d=6144, n_q_heads=2, n_kv_heads=2, head_dim=64, ffn=512,
                                      vocab=1000, ctx=40, K=12),
    # no q/k norm, 8 heads per K/V head (several query-tile groups), K 12
    "wide_group": ds.scaled_config("C2", d=1024, n_q_heads=8, n_kv_heads=1, head_dim=128, ffn=1024,
                                   vocab=4096, ctx=257, K=12, qk_norm=False),
}


def _run(cfg, seed, n_cached_list=(0,), K=None, check_intermediates=False, tol=None):
    K = cfg.K if K is None else K
    ctx, W = make_context(cfg, seed)
    hidden = ds.make_hidden(cfg, seed + 1)
    ref, inter = odf.draft_forward(cfg, W, hidden, K, return_intermediates=True)
    h_dev = hidden_to_device(cfg, hidden)
    tol = tol or (BF16_TOL if cfg.dtype == "bf16" else F32_TOL)
    first = None
    for n_cached in n_cached_list:
        if n_cached == 0:
            ctx.reset()
        out = ctx.draft_forward(h_dev, cfg.ctx, K, n_cached=n_cached).cpu().numpy()
        if check_intermediates:
            n = cfg.ctx
            M = (n - n_cached) + K - 1
            M = M if M <= 16 else K
            a_gpu = ctx.debug_read("xn", M, cfg.d)
            np.testing.assert_allclose(a_gpu, inter["a"][n + K - 1 - M:], rtol=1e-3, atol=1e-3)
            for name, key in (("att_out", "o"), ("y", "y"), ("hmid", None), ("u", "u")):
                if key is None:
                    continue
                got = ctx.debug_read(name, K, inter[key].shape[1])
                scale = np.abs(inter[key]).max()
                assert np.abs(got - inter[key]).max() <= 2e-2 * scale + 1e-3, name
        ok, msg = logits_close(out, ref, **tol)
        assert ok, f"{cfg.name} n_cached={n_cached}: {msg}"
        if first is None:
            first = out
        else:
            # K/V of a row depend on that row only: cold and warm calls agree bit for bit
            np.testing.assert_array_equal(out, first)
    ctx.close()
    return ref


def test_c1_fp32_cold_and_warm_match_oracle():
    cfg = ds.get_config("C1")
    n = cfg.ctx
    _run(cfg, 1000, n_cached_list=(0, n - 1, n - 4, 10, 0), check_intermediates=True)


@pytest.mark.parametrize("name", sorted(SMALL_BF16))
def test_small_bf16_shapes_match_oracle(name):
    cfg = SMALL_BF16[name]
    n = cfg.ctx
    _run(cfg, 2000, n_cached_list=(0, n - 1, n - 3, 0), check_intermediates=True)


def test_fp32_variants_qknorm_and_short_contexts():
    for i, over in enumerate((dict(qk_norm=True), dict(ctx=1, K=4), dict(ctx=2, K=1),
                              dict(ctx=129, K=4, head_dim=128, n_q_heads=4, n_kv_heads=2))):
        cfg = ds.scaled_config("C1", **over)
        _run(cfg, 3000 + i)


def test_shorter_draft_and_longer_capacity():
    """K below max_K and a context shorter than max_ctx use the same buffers."""
    cfg = SMALL_BF16["mid128"]
    ctx, W = make_context(cfg, 2100)
    for n, K in ((301, 8), (40, 3), (200, 1)):
        hidden = ds.make_hidden(cfg, 2101 + n, n=n)
        ref = odf.draft_forward(cfg, W, hidden, K)
        ctx.reset()
        out = ctx.draft_forward(hidden_to_device(cfg, hidden), n, K).cpu().numpy()
        ok, msg = logits_close(out, ref, **BF16_TOL)
        assert ok, (n, K, msg)
    ctx.close()


def test_longest_context_the_library_accepts():
    """max_ctx + max_K = 32768 (256 key chunks per K/V head): cold call, warm call, oracle."""
    cfg = ds.scaled_config("C2", d=256, n_q_heads=4, n_kv_heads=2, head_dim=128, ffn=512,
                           vocab=1024, ctx=32760, K=8)
    ctx, W = make_context(cfg, 2150)
    hidden = ds.make_hidden(cfg, 2151)
    h_dev = hidden_to_device(cfg, hidden)
    n = cfg.ctx
    cold = ctx.draft_forward(h_dev, n, cfg.K, n_cached=0).cpu().numpy()
    ok, msg = logits_close(cold, odf.draft_forward(cfg, W, hidden, cfg.K), **BF16_TOL)
    assert ok, msg
    warm = ctx.draft_forward(h_dev, n, cfg.K, n_cached=n - 3).cpu().numpy()
    np.testing.assert_array_equal(warm, cold)
    ctx.close()


def test_growing_context_like_decoding():
    """Successive calls with a growing prefix reuse cached rows (accepted-token appends)."""
    cfg = SMALL_BF16["tiny64"]
    ctx, W = make_context(cfg, 2200)
    hidden = ds.make_hidden(cfg, 2201)
    h_dev = hidden_to_device(cfg, hidden)
    cached = 0
    for n in (20, 21, 25, 26, 60, 70):
        out = ctx.draft_forward(h_dev, n, cfg.K, n_cached=cached).cpu().numpy()
        ref = odf.draft_forward(cfg, W, hidden[:n], cfg.K)
        ok, msg = logits_close(out, ref, **BF16_TOL)
        assert ok, (n, msg)
        cached = n
    ctx.close()


def test_batched_ragged_sequences():
    cfg = ds.scaled_config("C2", d=256, n_q_heads=4, n_kv_heads=2, head_dim=128, ffn=512,
                           vocab=1024, ctx=90, K=4, batch=3)
    ctx, W = make_context(cfg, 2300)
    lens = [90, 17, 33]
    hiddens = [ds.make_hidden(cfg, 2301 + b, n=lens[b]) for b in range(3)]
    devs = [hidden_to_device(cfg, h) for h in hiddens]
    out = ctx.draft_forward_batched(devs, lens, [0, 0, 0], cfg.K).cpu().numpy()
    for b in range(3):
        ref = odf.draft_forward(cfg, W, hiddens[b], cfg.K)
        ok, msg = logits_close(out[b], ref, **BF16_TOL)
        assert ok, (b, msg)
    ctx.close()


@pytest.mark.parametrize("batch,K,over", [
    (6, 8, dict(d=512, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn=1536, vocab=8200, ctx=150)),
    (16, 8, dict(d=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=5632, vocab=1000, ctx=120)),
    (2, 3, dict(d=1024, n_q_heads=8, n_kv_heads=1, head_dim=128, ffn=1024, vocab=40000, ctx=70,
                qk_norm=False)),
    (20, 2, dict(d=256, n_q_heads=4, n_kv_heads=4, head_dim=64, ffn=512, vocab=2048, ctx=40)),
    # long ragged contexts with one and two query tiles: several chunk units per attention
    # workgroup, pairs that end inside a run, four and two key sub-ranges merged in the workgroup
    (16, 4, dict(d=256, n_q_heads=2, n_kv_heads=2, head_dim=128, ffn=512, vocab=1024, ctx=2300)),
    (12, 8, dict(d=256, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn=512, vocab=1024, ctx=3000)),
])
def test_batched_multi_row_kernel_matches_oracle_cold_and_warm(batch, K, over):
    """The batched entry point runs every projection on the multi-row MFMA kernel: 48 and 128
    row passes, ragged vocab / strip tails, k-chunked matrices, more sequences than one pass
    holds; a warm call (cached prefix) reproduces the cold call bit for bit."""
    cfg = ds.scaled_config("C2", K=K, batch=batch, **over)
    ctx, W = make_context(cfg, 2500)
    rng = np.random.default_rng(2500 + batch)
    lens = [int(v) for v in rng.integers(5, cfg.ctx + 1, size=batch)]
    lens[0] = cfg.ctx
    hiddens = [ds.make_hidden(cfg, 2501 + b, n=lens[b]) for b in range(batch)]
    devs = [hidden_to_device(cfg, h) for h in hiddens]
    cold = ctx.draft_forward_batched(devs, lens, [0] * batch, K).cpu().numpy()
    for b in range(batch):
        ref = odf.draft_forward(cfg, W, hiddens[b], K)
        ok, msg = logits_close(cold[b], ref, **BF16_TOL)
        assert ok, (b, lens[b], msg)
    # shorter prefixes first, then the full ones with those rows cached
    part = [max(1, n - 1 - (b % 4)) for b, n in enumerate(lens)]
    for b in range(batch):
        ctx.reset(b)
    ctx.draft_forward_batched(devs, part, [0] * batch, K)
    warm = ctx.draft_forward_batched(devs, lens, part, K).cpu().numpy()
    np.testing.assert_array_equal(warm, cold)
    ctx.close()


def test_large_magnitude_hidden_states_without_qk_norm():
    """Hidden states 1024 times larger than the presets' (and 1/1024 of them), q/k norm off: every
    projection input is RMS-normalised, so the fp16 intermediates of the bf16 path (rotated q, the
    K/V buffers, the packed operands of the batched call) stay in range and the logits stay within
    tolerance, on both entry points."""
    cfg = ds.scaled_config("C2", d=512, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn=1536,
                           vocab=4096, ctx=150, K=8, qk_norm=False, batch=3)
    ctx, W = make_context(cfg, 2600)
    for scale in (1024.0, 1.0 / 1024.0):
        lens = [150, 40, 97]
        hiddens = [ds.f32_to_bf16_bits(ds.bf16_bits_to_f32(ds.make_hidden(cfg, 2601 + b, n=lens[b])) * scale)
                   for b in range(3)]
        devs = [hidden_to_device(cfg, h) for h in hiddens]
        refs = [odf.draft_forward(cfg, W, h, cfg.K) for h in hiddens]
        for b in range(3):
            ctx.reset(b)
        single = ctx.draft_forward(devs[0], lens[0], cfg.K).cpu().numpy()
        ok, msg = logits_close(single, refs[0], **BF16_TOL)
        assert ok, (scale, msg)
        for b in range(3):
            ctx.reset(b)
        out = ctx.draft_forward_batched(devs, lens, [0, 0, 0], cfg.K).cpu().numpy()
        for b in range(3):
            ok, msg = logits_close(out[b], refs[b], **BF16_TOL)
            assert ok, (scale, b, msg)
    ctx.close()


def test_error_statuses():
    import torch
    import paper_2601_19278_amd as dart
    cfg = SMALL_BF16["tiny64"]
    ctx, _ = make_context(cfg, 2400)
    h = hidden_to_device(cfg, ds.make_hidden(cfg, 2401))
    out = torch.full((cfg.K, cfg.vocab), 7.0, device="cuda")
    for kwargs, status in ((dict(ctx_len=cfg.ctx + 1, K=cfg.K), 2), (dict(ctx_len=10, K=cfg.K + 1), 1),
                           (dict(ctx_len=0, K=1), 1), (dict(ctx_len=10, K=2, n_cached=5), 5),
                           (dict(ctx_len=10, K=2, seq=3), 1)):
        with pytest.raises(dart.DartError) as ei:
            ctx.draft_forward(h, out=out, **kwargs)
        assert ei.value.status == status, kwargs
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())                      # outputs untouched on error
    ctx.draft_forward(h, 10, 2)
    with pytest.raises(dart.DartError) as ei:
        ctx.draft_forward(h, 10, 2, n_cached=10)         # the last prefix row is always a query row
    assert ei.value.status == 5
    ctx.draft_forward(h, 12, 2, n_cached=10)
    ctx.close()


def test_c2_full_size_matches_oracle():
    cfg = ds.get_config("C2")
    _run(cfg, 1000 * 2, n_cached_list=(0, cfg.ctx - 1, cfg.ctx - 4))


def test_c4_headline_full_size_matches_oracle():
    cfg = ds.get_config("C4")
    _run(cfg, 1000 * 4, n_cached_list=(0, cfg.ctx - 1, cfg.ctx - 4))


def test_c3_full_size_matches_oracle():
    cfg = ds.get_config("C3")
    _run(cfg, 1000 * 3, n_cached_list=(0, cfg.ctx - 1, cfg.ctx - 4))


def test_c5_batched_ragged_full_size_sampled_sequences_match_oracle():
    """Preset C5: 16 ragged sequences through dart_draft_forward_batched; the oracle checks the
    shortest, the median and the longest sequence (all K x vocab logits of each)."""
    from dart_synth.tensors import make_ragged_lengths
    cfg = ds.get_config("C5")
    ctx, W = make_context(cfg, 5000)
    lens = make_ragged_lengths(cfg, 5001).tolist()
    hiddens = [ds.make_hidden(cfg, 5002 + b, n=lens[b]) for b in range(cfg.batch)]
    devs = [hidden_to_device(cfg, h) for h in hiddens]
    out = ctx.draft_forward_batched(devs, lens, [0] * cfg.batch, cfg.K).cpu().numpy()
    order = np.argsort(lens)
    for b in (int(order[0]), int(order[len(order) // 2]), int(order[-1])):
        ref = odf.draft_forward(cfg, W, hiddens[b], cfg.K)
        ok, msg = logits_close(out[b], ref, **BF16_TOL)
        assert ok, f"sequence {b} (n={lens[b]}): {msg}"
    # a second, warm batched call (one new token per sequence) reproduces a cold call bit for bit
    lens2 = [min(n + 1, cfg.ctx) for n in lens]
    hid2 = [ds.make_hidden(cfg, 5002 + b, n=lens2[b]) for b in range(cfg.batch)]
    for b in range(cfg.batch):
        assert np.array_equal(hid2[b][: lens[b]], hiddens[b])
    dev2 = [hidden_to_device(cfg, h) for h in hid2]
    warm = ctx.draft_forward_batched(dev2, lens2, lens, cfg.K).cpu().numpy()
    for b in range(cfg.batch):
        ctx.reset(b)
    cold = ctx.draft_forward_batched(dev2, lens2, [0] * cfg.batch, cfg.K).cpu().numpy()
    np.testing.assert_array_equal(warm, cold)
    ctx.close()
