"""Helpers shared by the GPU parity tests (no arithmetic of the method lives here)."""
import numpy as np

import dart_synth as ds


def hidden_to_device(cfg, hidden_np):
    import torch
    import paper_2601_19278_amd as dart
    if cfg.dtype == "bf16":
        return dart.bf16_bits_to_tensor(hidden_np)
    return torch.from_numpy(hidden_np).cuda()


def make_context(cfg, seed, max_ctx=None, max_K=None, max_batch=None):
    import paper_2601_19278_amd as dart
    weights = ds.make_weights(cfg, seed, max_K=max_K)
    ctx = dart.DraftContext(cfg, weights, max_ctx=max_ctx, max_K=max_K, max_batch=max_batch)
    return ctx, weights


def logits_close(gpu, ref, atol, rtol):
    """max-abs / relative criterion |g - o| <= atol + rtol |o|; returns (ok, worst excess info)."""
    gpu = np.asarray(gpu, dtype=np.float64)
    err = np.abs(gpu - ref)
    bound = atol + rtol * np.abs(ref)
    worst = np.unravel_index(np.argmax(err - bound), err.shape)
    return bool((err <= bound).all()), f"max|err|={err.max():.3e} at {worst}: gpu={gpu[worst]:.6f} ref={ref[worst]:.6f}"
