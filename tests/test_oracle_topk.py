"""Pins for the oracle's candidate extraction (Alg. 1 Top-k_i / s_logit, App. D)."""
import numpy as np
import torch

from oracle import topk as otk


def _rows(R, V, seed):
    return np.random.default_rng(seed).standard_normal((R, V)).astype(np.float32) * 3


def test_matches_library_topk_and_log_softmax():
    logits = _rows(5, 1000, 0)
    ids, scores = otk.topk_rows(logits, 7, 1e-9)
    t = torch.from_numpy(logits).double()
    ref_val, ref_idx = torch.topk(t, 7, dim=1)
    np.testing.assert_array_equal(ids, ref_idx.numpy())
    lsm = torch.log_softmax(t, dim=1).gather(1, ref_idx).numpy()
    np.testing.assert_allclose(scores, np.log(np.exp(lsm) + 1e-9), rtol=2e-7, atol=1e-7)


def test_k_equals_vocab_is_a_permutation_and_probabilities_sum_to_one():
    V, eps = 257, 1e-6
    logits = _rows(1, V, 1)
    ids, scores = otk.topk_rows(logits, V, eps)
    assert sorted(ids[0].tolist()) == list(range(V))
    assert np.all(np.diff(logits[0][ids[0]]) <= 0)
    np.testing.assert_allclose(np.exp(scores[0].astype(np.float64)).sum(), 1 + V * eps, rtol=1e-6)


def test_k1_is_argmax_and_brute_force_agrees():
    logits = _rows(4, 300, 2)
    ids, _ = otk.topk_rows(logits, 1, 1e-9)
    np.testing.assert_array_equal(ids[:, 0], logits.argmax(axis=1))
    ids3, _ = otk.topk_rows(logits, 3, 1e-9)
    for r in range(4):
        row = logits[r].tolist()
        picked = []
        for _ in range(3):                       # repeated max extraction, first index wins
            j = max(range(len(row)), key=lambda i: (row[i], -i))
            picked.append(j)
            row[j] = float("-inf")
        assert ids3[r].tolist() == picked


def test_ties_resolve_to_lower_token_id_and_signed_zero_is_a_tie():
    logits = np.zeros((1, 10), dtype=np.float32)
    logits[0, [7, 2, 5]] = 4.0
    logits[0, 3] = -0.0
    ids, scores = otk.topk_rows(logits, 5, 1e-9)
    assert ids[0].tolist() == [2, 5, 7, 0, 1]
    assert scores[0, 0] == scores[0, 1] == scores[0, 2]


def test_scores_never_positive_and_eps_floor():
    logits = np.array([[50.0, 0.0, -80.0]], dtype=np.float32)
    ids, scores = otk.topk_rows(logits, 3, 1e-9)
    assert ids[0].tolist() == [0, 1, 2]
    assert scores[0, 0] == 0.0                                   # log(1 + eps) clamps to 0
    np.testing.assert_allclose(scores[0, 2], np.log(np.exp(-130.0) + 1e-9), rtol=1e-6)
    np.testing.assert_allclose(scores[0, 1], np.log(np.exp(-50.0) + 1e-9), rtol=1e-6)


def test_log_sum_exp_closed_form():
    row = np.log(np.array([1.0, 2.0, 3.0, 4.0]))
    np.testing.assert_allclose(otk.log_sum_exp(row), np.log(10.0), rtol=1e-14)
    np.testing.assert_allclose(otk.log_sum_exp(np.full(8, 1000.0)), 1000.0 + np.log(8.0), rtol=1e-14)
