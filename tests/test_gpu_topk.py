"""GPU parity: dart_topk against the oracle's full-sort top-k on the same logits buffer."""
import numpy as np
import pytest

import dart_synth as ds
from oracle import topk as otk
from util_gpu import make_context

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    # a context is only needed for its top-k workspace: tiny layer, full-size vocabulary
    cfg = ds.scaled_config("C1", vocab=151936, K=16, batch=1)
    c, _ = make_context(cfg, 50, max_K=16)
    yield c
    c.close()


def _check(ctx, logits, k, eps=1e-9):
    import torch
    ids, scores = ctx.topk(torch.from_numpy(logits).cuda(), k, eps)
    ids, scores = ids.cpu().numpy(), scores.cpu().numpy()
    ref_ids, ref_scores = otk.topk_rows(logits, k, eps)
    np.testing.assert_array_equal(ids, ref_ids)              # ids and their order: bit-exact
    np.testing.assert_allclose(scores, ref_scores, rtol=0, atol=1e-5)
    assert (scores <= 0).all()


@pytest.mark.parametrize("V,k,rows", [(151936, 10, 8), (151936, 25, 8), (8192, 4, 4), (4096, 1, 3),
                                       (4097, 64, 2), (1000, 7, 16), (5, 5, 1), (100000, 64, 5)])
def test_random_rows(ctx, V, k, rows):
    rng = np.random.default_rng(V * 131 + k)
    logits = (rng.standard_normal((rows, V)) * 1.5).astype(np.float32)
    _check(ctx, logits, k)


def test_peaked_rows_and_eps(ctx):
    rng = np.random.default_rng(7)
    logits = (rng.standard_normal((4, 50000)) * 8).astype(np.float32)   # low-entropy rows
    _check(ctx, logits, 10, eps=1e-9)
    _check(ctx, logits, 10, eps=1e-4)


def test_ties_and_signed_zero(ctx):
    logits = np.zeros((2, 9000), dtype=np.float32)
    logits[0, [8999, 4096, 4095, 17]] = 3.0          # ties across chunk borders
    logits[0, 100] = -0.0
    logits[1, :] = -1.0
    logits[1, [5000, 2]] = -0.0
    logits[1, 7000] = 0.0
    _check(ctx, logits, 8)


def test_repeat_runs_are_bit_identical(ctx):
    import torch
    rng = np.random.default_rng(9)
    logits = torch.from_numpy(rng.standard_normal((8, 151936)).astype(np.float32)).cuda()
    first = [t.clone() for t in ctx.topk(logits, 10)]
    for _ in range(20):
        ids, scores = ctx.topk(logits, 10)
        assert torch.equal(ids, first[0]) and torch.equal(scores, first[1])


def test_128_rows_of_a_batched_step_and_heavy_ties():
    """The batched step's 128 logit rows in one call; rows whose values tie in large groups
    (more candidates at the selection threshold than the compaction buffer holds)."""
    cfg = ds.scaled_config("C1", vocab=151936, K=16, batch=8)
    c, _ = make_context(cfg, 51, max_K=16)
    rng = np.random.default_rng(11)
    logits = (rng.standard_normal((128, 151936)) * 2).astype(np.float32)
    logits[5] = np.round(logits[5])                  # ~10 distinct values: ties by the thousand
    logits[6] = 0.25
    logits[7, ::2] = 4.0
    _check(c, logits, 10)
    _check(c, logits[:9], 64)
    # more than 16 rows take the two-launch form: its edge shapes, and repeatability
    _check(c, logits[:40], 64)
    _check(c, np.ascontiguousarray(logits[:17, :4097]), 64)
    _check(c, np.ascontiguousarray(logits[:33, :5]), 5)
    _check(c, np.ascontiguousarray(logits[:128, :1000]), 7)
    import torch
    dev = torch.from_numpy(logits).cuda()
    first = [t.clone() for t in c.topk(dev, 10)]
    for _ in range(5):
        ids, scores = c.topk(dev, 10)
        assert torch.equal(ids, first[0]) and torch.equal(scores, first[1])
    c.close()


def test_vocabulary_with_more_chunks_than_merge_registers():
    """More chunk winners (chunks x k) than the row merge holds in registers: it re-reads them."""
    cfg = ds.scaled_config("C1", vocab=170000, K=4, batch=1)
    c, _ = make_context(cfg, 52, max_K=4)
    rng = np.random.default_rng(12)
    logits = (rng.standard_normal((3, 170000)) * 2).astype(np.float32)
    logits[2, 169990:] = 9.0                          # winners in the ragged last chunk, tied
    _check(c, logits, 10)
    _check(c, logits, 1)
    _check(c, logits, 64)                             # 42 chunks x 64 > 2560: the re-read path
    c.close()


def test_error_statuses(ctx):
    import torch
    import paper_2601_19278_amd as dart
    logits = torch.zeros((2, 100), device="cuda")
    for k in (0, 65, 101):
        with pytest.raises(dart.DartError) as ei:
            ctx.topk(logits, k)
        assert ei.value.status == 1
    with pytest.raises(dart.DartError) as ei:
        ctx.topk(torch.zeros((17, 100), device="cuda"), 3)
    assert ei.value.status == 2
