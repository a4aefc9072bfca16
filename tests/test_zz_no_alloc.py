"""GPU test of dart_topk_static, the top-k entry point for callers that cannot allocate: it
must give what dart_topk gives (bit for bit: same kernels, another workspace) and what the
oracle's full sort gives, on two calls in a row, the second with a smaller input (the shared
workspace keeps the first call's contents)."""
import numpy as np
import pytest

import dart_synth as ds
from oracle import topk as otk
from util_gpu import make_context

pytestmark = pytest.mark.gpu


def _both(ctx, logits_np, k, eps=1e-9):
    import torch
    import paper_2601_19278_amd as dart
    dev = torch.from_numpy(logits_np).cuda()
    rows = logits_np.shape[0]
    out = (torch.full((rows, k), -7, dtype=torch.int32, device="cuda"),
           torch.full((rows, k), 7.0, dtype=torch.float32, device="cuda"))
    ids_s, sc_s = dart.topk_static(dev, k, eps, out=out)
    ids_c, sc_c = ctx.topk(dev, k, eps)
    torch.cuda.synchronize()
    assert torch.equal(ids_s, ids_c) and torch.equal(sc_s, sc_c)
    ref_ids, ref_scores = otk.topk_rows(logits_np, k, eps)
    np.testing.assert_array_equal(ids_s.cpu().numpy(), ref_ids)
    np.testing.assert_allclose(sc_s.cpu().numpy(), ref_scores, rtol=0, atol=1e-5)


def test_static_workspace_topk_matches_context_topk_and_oracle():
    import torch
    import paper_2601_19278_amd as dart
    cfg = ds.scaled_config("C1", vocab=151936, K=16, batch=8)
    ctx, _ = make_context(cfg, 60, max_K=16)
    rng = np.random.default_rng(61)
    big = (rng.standard_normal((128, 151936)) * 2).astype(np.float32)     # every workspace cell
    big[3, ::3] = 5.0                                                      # heavy ties
    _both(ctx, big, 10)
    small = (rng.standard_normal((5, 9000)) * 2).astype(np.float32)       # then a smaller input
    small[0, [8999, 4096, 4095, 17]] = 3.0                                 # ties across chunk borders
    _both(ctx, small, 64)
    _both(ctx, np.ascontiguousarray(big[:8]), 10)                          # the draft step's shape
    _both(ctx, np.ascontiguousarray(small[:1, :5]), 5)
    # limits: one cell too many is refused with outputs untouched; argument errors as dart_topk
    lib = dart.load_library()
    dev = torch.zeros((129, 151936), device="cuda")
    ids = torch.full((129, 4), -7, dtype=torch.int32, device="cuda")
    sc = torch.full((129, 4), 7.0, device="cuda")
    assert lib.dart_topk_static(dev.data_ptr(), 129, 151936, 4, 1e-9, ids.data_ptr(), sc.data_ptr(), None) == 2
    assert lib.dart_topk_static(dev.data_ptr(), 2, 100, 0, 1e-9, ids.data_ptr(), sc.data_ptr(), None) == 1
    assert lib.dart_topk_static(dev.data_ptr(), 2, 100, 101, 1e-9, ids.data_ptr(), sc.data_ptr(), None) == 1
    assert lib.dart_topk_static(None, 2, 100, 3, 1e-9, ids.data_ptr(), sc.data_ptr(), None) == 1
    torch.cuda.synchronize()
    assert bool((ids == -7).all()) and bool((sc == 7.0).all())
    ctx.close()
