"""Host-side checks (no GPU): the C-ABI library loads, exports every symbol the header
declares, and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import dart_synth as ds

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def dart():
    import paper_2601_19278_amd as pkg
    if not os.path.exists(pkg.library_path()):
        from paper_2601_19278_amd import build
        build.build(verbose=False)
    return pkg


def _declared(header_name, skip_ifdef=None):
    header = open(os.path.join(ROOT, "include", header_name)).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    if skip_ifdef:
        header = re.sub(r"#ifdef %s\b.*?#endif" % skip_ifdef, "", header, flags=re.S)
    return set(re.findall(r"\b(dart_[a-z_]+)\s*\(", header))


def test_header_symbols_are_exported(dart):
    declared = _declared("dart.h")
    assert declared == set(dart.EXPORTED_SYMBOLS)
    assert not any("debug" in name for name in declared)          # diagnostics live elsewhere
    debug = _declared("dart_debug.h", skip_ifdef="DART_TUNING")
    assert debug == set(dart.DEBUG_SYMBOLS)
    lib = dart.load_library()
    for name in declared | debug:
        assert hasattr(lib, name), name
    assert not hasattr(lib, "dart_debug_set")        # product build: launch tunables are constants
    assert lib.dart_status_str(0) == b"ok"
    assert lib.dart_status_str(5) == b"invalid call sequence"


def test_create_rejects_bad_configs_without_a_device(dart):
    cfg = ds.scaled_config("C1", d=64, n_q_heads=2, n_kv_heads=2, head_dim=64, ffn=64, vocab=32,
                           ctx=8, K=2)
    W = ds.make_weights(cfg, 1)
    for over in (dict(head_dim=32), dict(n_q_heads=3), dict(K=17), dict(vocab=0), dict(d=66)):
        bad = ds.scaled_config("C1", **{**dict(d=64, n_q_heads=2, n_kv_heads=2, head_dim=64, ffn=64,
                                               vocab=32, ctx=8, K=2), **over})
        with pytest.raises(dart.DartError) as ei:
            dart.DraftContext(bad, W)
        assert ei.value.status == 1, over
    W2 = dict(W)
    W2["wq"] = None
    with pytest.raises(dart.DartError) as ei:
        dart.DraftContext(cfg, W2)
    assert ei.value.status == 1
    bf = ds.scaled_config("C2", d=16416, n_q_heads=2, n_kv_heads=2, head_dim=64, ffn=64, vocab=32,
                          ctx=8, K=2)
    with pytest.raises(dart.DartError) as ei:        # d beyond what the row kernels hold
        dart.DraftContext(bf, {k: np.zeros(1, np.uint16) for k in ds.WEIGHT_NAMES})
    assert ei.value.status == 1


def test_ngram_and_prune_argument_checks(dart):
    lib = dart.load_library()
    h = C.c_void_p()
    keys = np.array([[1, 2]], np.int32)
    ids = np.array([[3, 4]], np.int32)
    cnt = np.array([[1, 1]], np.int32)
    args = (keys.ctypes.data, ids.ctypes.data, cnt.ctypes.data)
    assert lib.dart_ngram_create(4, 1, 2, *args, 1e-9, C.byref(h)) == 1      # N must be 2 or 3
    assert lib.dart_ngram_create(3, 1, 65, *args, 1e-9, C.byref(h)) == 1     # S <= 64
    assert lib.dart_ngram_create(3, 1, 2, None, None, None, 1e-9, C.byref(h)) == 1
    neg = np.array([[-1, 2]], np.int32)
    assert lib.dart_ngram_create(3, 1, 2, neg.ctypes.data, args[1], args[2], 1e-9, C.byref(h)) == 1
    # a used successor with a negative id, a successor repeated within its row, a negative count
    for bad_ids, bad_cnt in (([[3, -1]], [[1, 1]]), ([[3, 3]], [[1, 2]]), ([[3, 4]], [[1, -1]])):
        bi, bc = np.array(bad_ids, np.int32), np.array(bad_cnt, np.int32)
        assert lib.dart_ngram_create(3, 1, 2, args[0], bi.ctypes.data, bc.ctypes.data, 1e-9, C.byref(h)) == 1
    dup = np.array([[1, 2], [1, 2]], np.int32)                               # the same context twice
    two = np.array([[3, 4], [5, 6]], np.int32)
    one = np.ones((2, 2), np.int32)
    assert lib.dart_ngram_create(3, 2, 2, dup.ctypes.data, two.ctypes.data, one.ctypes.data, 1e-9, C.byref(h)) == 1
    # pruning parameters outside the range in which Alg. 1's top-theta set is a tree
    P = dart.binding._PruneParams
    buf = np.zeros(64, np.int32)
    ptr = buf.ctypes.data           # never dereferenced: the parameter check comes first
    for w_ng, decay, pw in ((-0.5, 0.9, 0.7), (0.5, 0.0, 0.7), (0.5, -0.9, 0.7), (0.5, 0.9, float("nan")),
                            (float("inf"), 0.9, 0.7), (0.5, float("nan"), 0.7)):
        p = P(2, 2, 4, w_ng, decay, pw)
        assert lib.dart_tree_prune(1, ptr, ptr, 2, ptr, ptr, C.byref(p), ptr, ptr, ptr, ptr, None) == 1
    assert lib.dart_tree_prune(1, None, None, 4, None, None, None, None, None, None, None, None) == 1
    assert lib.dart_topk(None, None, 1, 1, 1, 1e-9, None, None, None) == 1
    assert lib.dart_draft_forward(None, 0, None, 1, 0, 1, None, None) == 1
    assert lib.dart_reset(None, 0) == 1


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2601_19278_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.replace("no CPU fallback", ""), f
    for dirpath, _, files in os.walk(os.path.join(ROOT, "oracle")):
        for f in files:
            if f.endswith(".py"):
                assert "paper_2601_19278_amd" not in open(os.path.join(dirpath, f)).read(), f
