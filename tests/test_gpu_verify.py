"""GPU parity: dart_tree_verify_greedy against the oracle (bit-exact integer outputs)."""
import numpy as np
import pytest

import dart_synth as ds
from oracle import tree_prune as otp
from oracle import verify as ov
from oracle.ngram import NgramModel

pytestmark = pytest.mark.gpu


def _trees(seed0, count, K, k, w, budget):
    out = []
    for s in range(count):
        case = ds.make_prune_case(seed0 + s, vocab=2000, K=K, k=k, n_gram=3, S=16)
        model = NgramModel(3, case.table.keys, case.table.succ_ids, case.table.succ_counts, 1e-9)
        out.append(otp.tree_prune(case.ids, case.scores, case.ctx_tail, model,
                                  otp.PruneParams(k=k, beam_w=w, budget=budget)))
    return out


@pytest.mark.parametrize("K,k,w,budget,path_cap", [(8, 10, 20, 60, 17), (16, 6, 8, 128, 17),
                                                    (3, 2, 2, 5, 2), (1, 1, 1, 1, 1), (8, 4, 4, 70, 9)])
def test_positions_and_acceptance_match_oracle(K, k, w, budget, path_cap):
    import torch
    import paper_2601_19278_amd as dart
    B = 37
    trees = _trees(8000 + budget, B, K, k, w, budget)
    rng = np.random.default_rng(budget)
    tn = rng.integers(0, 2000, size=(B, budget)).astype(np.int32)
    for b, tr in enumerate(trees):                   # plant matching edges along random paths
        for i in range(tr.n_nodes):
            kids = [c for c in range(tr.n_nodes) if tr.parents[c] == i]
            if kids and rng.random() < 0.8:
                tn[b, i] = tr.tokens[kids[rng.integers(len(kids))]]
    ctx_len = rng.integers(1, 5000, size=B).astype(np.int32)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    pos, path, n_acc, nxt = dart.tree_verify_greedy(
        dev(np.stack([t.tokens for t in trees])), dev(np.stack([t.parents for t in trees])),
        dev(np.array([t.n_nodes for t in trees], np.int32)), dev(ctx_len), dev(tn), path_cap=path_cap)
    torch.cuda.synchronize()
    pos, path, n_acc, nxt = (x.cpu().numpy() for x in (pos, path, n_acc, nxt))
    for b, tr in enumerate(trees):
        depth = ov.tree_positions(tr.parents, tr.n_nodes)
        np.testing.assert_array_equal(pos[b], np.where(depth >= 0, depth + ctx_len[b], -1))
        ref_path, ref_next = ov.accept_greedy(tr.tokens, tr.parents, tr.n_nodes, tn[b])
        if len(ref_path) > path_cap:                 # the walk is cut at path_cap nodes
            ref_path = ref_path[:path_cap]
            ref_next = tn[b, ref_path[-1]]
        assert n_acc[b] == len(ref_path) - 1
        assert path[b, :len(ref_path)].tolist() == ref_path and (path[b, len(ref_path):] == -1).all()
        assert nxt[b] == ref_next


def test_positions_only_and_argument_errors():
    import torch
    import paper_2601_19278_amd as dart
    tr = _trees(8100, 1, 8, 10, 20, 60)[0]
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    tok, par, nn = dev(tr.tokens[None]), dev(tr.parents[None]), dev(np.array([tr.n_nodes], np.int32))
    pos, path, n_acc, nxt = dart.tree_verify_greedy(tok, par, nn)
    torch.cuda.synchronize()
    assert path is None and n_acc is None and nxt is None
    depth = ov.tree_positions(tr.parents, tr.n_nodes)
    np.testing.assert_array_equal(pos.cpu().numpy()[0], depth)
    lib = dart.load_library()
    assert lib.dart_tree_verify_greedy(1, None, par.data_ptr(), nn.data_ptr(), 60, None, pos.data_ptr(),
                                       None, 17, None, None, None, None) == 1
    assert lib.dart_tree_verify_greedy(1, tok.data_ptr(), par.data_ptr(), nn.data_ptr(), 129, None,
                                       pos.data_ptr(), None, 17, None, None, None, None) == 1
    assert lib.dart_tree_verify_greedy(1, tok.data_ptr(), par.data_ptr(), nn.data_ptr(), 60, None,
                                       pos.data_ptr(), tok.data_ptr(), 17, None, None, None, None) == 1
