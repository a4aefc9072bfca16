"""ctypes marshalling for libdart.so -- names and arguments mirror include/dart.h."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

EXPORTED_SYMBOLS = (
    "dart_status_str", "dart_create", "dart_destroy", "dart_reset", "dart_draft_forward",
    "dart_draft_forward_topk", "dart_draft_forward_topk_batched", "dart_draft_forward_features_topk",
    "dart_draft_forward_features", "dart_draft_forward_features_batched",
    "dart_draft_forward_batched", "dart_topk", "dart_topk_static", "dart_ngram_create", "dart_ngram_destroy",
    "dart_ngram_set_backoff",
    "dart_tree_prune", "dart_tree_verify_greedy",
)
# include/dart_debug.h: diagnostics for this repository's tests and benchmark, not product API
DEBUG_SYMBOLS = ("dart_debug_read", "dart_debug_lm_head", "dart_debug_lm_head_select",
                 "dart_debug_lm_head_key", "dart_debug_stream_read")

DART_F32, DART_BF16 = 0, 1


class DartError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: status {status} ({_status_str(status)})")


class _Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("d", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "vocab",
                                         "max_ctx", "max_K", "max_batch", "dtype", "qk_norm")] + \
               [("rms_eps", C.c_float), ("rope_base", C.c_float), ("front_end", C.c_int32),
                ("feat_dim", C.c_int32)]


_WEIGHT_FIELDS = ("w_in_norm", "wq", "wk", "wv", "q_norm", "k_norm", "wo", "w_post_norm",
                  "w_gate", "w_up", "w_down", "w_final_norm", "w_lm", "mask_emb",
                  "w_fc", "embed", "w_emb_norm")


class _Weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _WEIGHT_FIELDS]


class _PruneParams(C.Structure):
    _fields_ = [("k", C.c_int32), ("beam_w", C.c_int32), ("budget", C.c_int32),
                ("w_ng", C.c_float), ("logit_decay", C.c_float), ("level_pow", C.c_float)]


@dataclass
class PruneParams:
    """Pruning hyper-parameters (paper App. D defaults: w = 20, theta = 59 -> budget 60)."""
    k: int
    beam_w: int = 20
    budget: int = 60
    w_ng: float = 0.5
    logit_decay: float = 0.9
    level_pow: float = 0.7


def library_path() -> str:
    return os.path.join(_HERE, "libdart.so")


def load_library() -> C.CDLL:
    """Load libdart.so; raises if it has not been built (no fallback path exists)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it with `python -m paper_2601_19278_amd.build`")
    # PyTorch ships its own HIP runtime (same SONAME as the system one).  Import it first so
    # that libdart.so binds to that copy; two HIP runtimes in one process cannot share the GPU.
    import torch  # noqa: F401
    lib = C.CDLL(path)
    vp, i32, i64, f32 = C.c_void_p, C.c_int, C.c_int64, C.c_float
    lib.dart_status_str.restype = C.c_char_p
    lib.dart_status_str.argtypes = [i32]
    lib.dart_create.argtypes = [C.POINTER(_Config), C.POINTER(_Weights), C.POINTER(vp)]
    lib.dart_destroy.argtypes = [vp]
    lib.dart_destroy.restype = None
    lib.dart_reset.argtypes = [vp, i32]
    lib.dart_draft_forward.argtypes = [vp, i32, vp, i32, i32, i32, vp, vp]
    lib.dart_draft_forward_topk.argtypes = [vp, i32, vp, i32, i32, i32, i32, f32, vp, vp, vp, vp]
    lib.dart_draft_forward_features.argtypes = [vp, i32, vp, vp, i32, i32, i32, vp, vp]
    lib.dart_draft_forward_features_topk.argtypes = [vp, i32, vp, vp, i32, i32, i32, i32, f32, vp, vp, vp, vp]
    lib.dart_draft_forward_batched.argtypes = [vp, i32, C.POINTER(vp), C.POINTER(C.c_int32),
                                               C.POINTER(C.c_int32), i32, vp, vp]
    lib.dart_draft_forward_topk_batched.argtypes = [vp, i32, C.POINTER(vp), C.POINTER(C.c_int32),
                                                    C.POINTER(C.c_int32), i32, i32, f32, vp, vp, vp, vp]
    lib.dart_draft_forward_features_batched.argtypes = [vp, i32, C.POINTER(vp), C.POINTER(vp),
                                                        C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                                        i32, vp, vp]
    lib.dart_topk.argtypes = [vp, vp, i32, i32, i32, f32, vp, vp, vp]
    lib.dart_topk_static.argtypes = [vp, i32, i32, i32, f32, vp, vp, vp]
    lib.dart_ngram_create.argtypes = [i32, i64, i32, vp, vp, vp, f32, C.POINTER(vp)]
    lib.dart_ngram_set_backoff.argtypes = [vp, i64, vp, vp, vp, f32]
    lib.dart_ngram_destroy.argtypes = [vp]
    lib.dart_ngram_destroy.restype = None
    lib.dart_tree_prune.argtypes = [i32, vp, vp, i32, vp, vp, C.POINTER(_PruneParams), vp, vp, vp,
                                    vp, vp]
    lib.dart_tree_verify_greedy.argtypes = [i32, vp, vp, vp, i32, vp, vp, vp, i32, vp, vp, vp, vp]
    lib.dart_debug_read.argtypes = [vp, C.c_char_p, vp, i64]
    lib.dart_debug_read.restype = i64
    lib.dart_debug_lm_head.argtypes = [vp, i32, i32, vp, vp]
    lib.dart_debug_lm_head_select.argtypes = [vp, i32, i32, vp, vp]
    lib.dart_debug_lm_head_key.argtypes = [vp, i32, i32, C.c_char_p, i32]
    lib.dart_debug_stream_read.argtypes = [vp, i64, i32, i32, vp, vp]
    if hasattr(lib, "dart_debug_set"):          # tuning builds (-DDART_TUNING) only
        lib.dart_debug_set.argtypes = [C.c_char_p, i32]
    _LIB = lib
    return lib


def _status_str(status: int) -> str:
    try:
        return load_library().dart_status_str(status).decode()
    except Exception:       # pragma: no cover
        return "?"


def _check(status: int, what: str) -> None:
    if status != 0:
        raise DartError(status, what)


def _torch():
    import torch
    return torch


def _stream_ptr(stream) -> int:
    torch = _torch()
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


def bf16_bits_to_tensor(bits: np.ndarray, device="cuda"):
    """uint16 bf16 bit patterns -> torch.bfloat16 tensor on `device` (no value change)."""
    torch = _torch()
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(device)


class DraftContext:
    """dart_ctx: device weights, draft K/V buffers and workspaces of one draft layer."""

    def __init__(self, cfg, weights: dict, max_ctx: int | None = None, max_K: int | None = None,
                 max_batch: int | None = None, feat_dim: int = 0):
        lib = load_library()
        self.dtype = DART_BF16 if cfg.dtype == "bf16" else DART_F32
        self.vocab, self.d = int(cfg.vocab), int(cfg.d)
        self.max_K = int(max_K if max_K is not None else cfg.K)
        self.max_ctx = int(max_ctx if max_ctx is not None else cfg.ctx)
        self.max_batch = int(max_batch if max_batch is not None else cfg.batch)
        c = _Config(d=cfg.d, n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads,
                    head_dim=cfg.head_dim, ffn=cfg.ffn, vocab=cfg.vocab, max_ctx=self.max_ctx,
                    max_K=self.max_K, max_batch=self.max_batch, dtype=self.dtype,
                    qk_norm=int(bool(cfg.qk_norm)), rms_eps=cfg.rms_eps, rope_base=cfg.rope_base,
                    front_end=int(feat_dim > 0), feat_dim=int(feat_dim))
        want = np.uint16 if self.dtype == DART_BF16 else np.float32
        keep, w = [], _Weights()
        for name in _WEIGHT_FIELDS:
            a = weights.get(name)
            if a is None:
                setattr(w, name, None)
                continue
            a = np.ascontiguousarray(a)
            if a.dtype != want:
                raise TypeError(f"weight {name}: expected {want}, got {a.dtype}")
            keep.append(a)
            setattr(w, name, a.ctypes.data)
        handle = C.c_void_p()
        _check(lib.dart_create(C.byref(c), C.byref(w), C.byref(handle)), "dart_create")
        self._h = handle
        self._lib = lib

    def close(self):
        if getattr(self, "_h", None):
            self._lib.dart_destroy(self._h)
            self._h = None

    __del__ = close

    def reset(self, seq: int = 0):
        _check(self._lib.dart_reset(self._h, seq), "dart_reset")

    def draft_forward(self, hidden, ctx_len: int, K: int, n_cached: int = 0, seq: int = 0,
                      out=None, stream=None):
        """dart_draft_forward: hidden is a CUDA tensor [>=ctx_len][d]; returns logits [K][vocab]."""
        torch = _torch()
        if out is None:
            out = torch.empty((K, self.vocab), dtype=torch.float32, device=hidden.device)
        _check(self._lib.dart_draft_forward(self._h, seq, hidden.data_ptr(), ctx_len, n_cached, K,
                                            out.data_ptr(), _stream_ptr(stream)),
               "dart_draft_forward")
        return out

    def draft_forward_topk(self, hidden, ctx_len: int, K: int, k: int, eps: float = 1e-9,
                           n_cached: int = 0, seq: int = 0, logits_out=None, out=None, stream=None):
        """dart_draft_forward_topk: the forward and the per-row top-k in one call; returns
        (ids [K][k] int32, scores [K][k] fp32); logits are written only if logits_out is given."""
        torch = _torch()
        if out is None:
            out = (torch.empty((K, k), dtype=torch.int32, device=hidden.device),
                   torch.empty((K, k), dtype=torch.float32, device=hidden.device))
        ids, scores = out
        _check(self._lib.dart_draft_forward_topk(self._h, seq, hidden.data_ptr(), ctx_len, n_cached, K, k,
                                                 eps, None if logits_out is None else logits_out.data_ptr(),
                                                 ids.data_ptr(), scores.data_ptr(), _stream_ptr(stream)),
               "dart_draft_forward_topk")
        return ids, scores

    def draft_forward_features(self, features, next_tokens, ctx_len: int, K: int, n_cached: int = 0,
                               seq: int = 0, out=None, stream=None):
        """dart_draft_forward_features: features CUDA [>=ctx_len][feat_dim], next_tokens CUDA int32
        [>=ctx_len]; returns logits [K][vocab]."""
        torch = _torch()
        if out is None:
            out = torch.empty((K, self.vocab), dtype=torch.float32, device=features.device)
        _check(self._lib.dart_draft_forward_features(self._h, seq, features.data_ptr(),
                                                     next_tokens.data_ptr(), ctx_len, n_cached, K,
                                                     out.data_ptr(), _stream_ptr(stream)),
               "dart_draft_forward_features")
        return out

    def draft_forward_features_topk(self, features, next_tokens, ctx_len: int, K: int, k: int,
                                    eps: float = 1e-9, n_cached: int = 0, seq: int = 0, logits_out=None,
                                    out=None, stream=None):
        """dart_draft_forward_features_topk: the front-end forward and the per-row top-k in one call;
        returns (ids [K][k] int32, scores [K][k] fp32); logits are written only if logits_out is given."""
        torch = _torch()
        if out is None:
            out = (torch.empty((K, k), dtype=torch.int32, device=features.device),
                   torch.empty((K, k), dtype=torch.float32, device=features.device))
        _check(self._lib.dart_draft_forward_features_topk(
            self._h, seq, features.data_ptr(), next_tokens.data_ptr(), ctx_len, n_cached, K, k, eps,
            logits_out.data_ptr() if logits_out is not None else None, out[0].data_ptr(), out[1].data_ptr(),
            _stream_ptr(stream)), "dart_draft_forward_features_topk")
        return out

    def draft_forward_batched(self, hiddens, ctx_lens, n_cached, K: int, out=None, stream=None):
        torch = _torch()
        B = len(hiddens)
        if out is None:
            out = torch.empty((B, K, self.vocab), dtype=torch.float32, device=hiddens[0].device)
        ptrs = (C.c_void_p * B)(*[h.data_ptr() for h in hiddens])
        lens = (C.c_int32 * B)(*[int(v) for v in ctx_lens])
        cached = (C.c_int32 * B)(*[int(v) for v in n_cached])
        _check(self._lib.dart_draft_forward_batched(self._h, B, ptrs, lens, cached, K,
                                                    out.data_ptr(), _stream_ptr(stream)),
               "dart_draft_forward_batched")
        return out

    def draft_forward_topk_batched(self, hiddens, ctx_lens, n_cached, K: int, k: int, eps: float = 1e-9,
                                   logits_out=None, out=None, stream=None):
        """dart_draft_forward_topk_batched: the batched forward and the per-row top-k in one call;
        returns (ids [B][K][k] int32, scores [B][K][k] fp32); logits are written only if
        logits_out ([B][K][vocab] fp32) is given."""
        torch = _torch()
        B = len(hiddens)
        if out is None:
            out = (torch.empty((B, K, k), dtype=torch.int32, device=hiddens[0].device),
                   torch.empty((B, K, k), dtype=torch.float32, device=hiddens[0].device))
        ptrs = (C.c_void_p * B)(*[h.data_ptr() for h in hiddens])
        lens = (C.c_int32 * B)(*[int(v) for v in ctx_lens])
        cached = (C.c_int32 * B)(*[int(v) for v in n_cached])
        _check(self._lib.dart_draft_forward_topk_batched(
            self._h, B, ptrs, lens, cached, K, k, eps,
            logits_out.data_ptr() if logits_out is not None else None, out[0].data_ptr(),
            out[1].data_ptr(), _stream_ptr(stream)), "dart_draft_forward_topk_batched")
        return out

    def draft_forward_features_batched(self, features, next_tokens, ctx_lens, n_cached, K: int,
                                       out=None, stream=None):
        """dart_draft_forward_features_batched: lists of CUDA tensors (features [n_b][feat_dim],
        next_tokens int32 [n_b]) and of lengths; returns logits [B][K][vocab]."""
        torch = _torch()
        B = len(features)
        if out is None:
            out = torch.empty((B, K, self.vocab), dtype=torch.float32, device=features[0].device)
        fptrs = (C.c_void_p * B)(*[f.data_ptr() for f in features])
        tptrs = (C.c_void_p * B)(*[t.data_ptr() for t in next_tokens])
        lens = (C.c_int32 * B)(*[int(v) for v in ctx_lens])
        cached = (C.c_int32 * B)(*[int(v) for v in n_cached])
        _check(self._lib.dart_draft_forward_features_batched(self._h, B, fptrs, tptrs, lens, cached,
                                                             K, out.data_ptr(), _stream_ptr(stream)),
               "dart_draft_forward_features_batched")
        return out

    def topk(self, logits, k: int, eps: float = 1e-9, stream=None, out=None):
        """dart_topk: logits CUDA fp32 [rows][vocab] -> (ids int32 [rows][k], scores fp32).
        `out` may carry preallocated (ids, scores) tensors."""
        torch = _torch()
        rows, vocab = logits.shape
        if out is None:
            ids = torch.empty((rows, k), dtype=torch.int32, device=logits.device)
            scores = torch.empty((rows, k), dtype=torch.float32, device=logits.device)
        else:
            ids, scores = out
        _check(self._lib.dart_topk(self._h, logits.data_ptr(), rows, vocab, k, eps, ids.data_ptr(),
                                   scores.data_ptr(), _stream_ptr(stream)), "dart_topk")
        return ids, scores

    def debug_lm_head(self, rows: int, out, stream=None, multi_row: int = 0):
        _check(self._lib.dart_debug_lm_head(self._h, rows, int(multi_row), out.data_ptr(),
                                            _stream_ptr(stream)), "dart_debug_lm_head")
        return out

    def debug_lm_head_select(self, rows: int, k: int, out=None, stream=None):
        _check(self._lib.dart_debug_lm_head_select(self._h, rows, k, out.data_ptr() if out is not None else None,
                                                   _stream_ptr(stream)), "dart_debug_lm_head_select")

    def debug_lm_head_key(self, rows: int, multi_row: int = 0) -> str:
        buf = C.create_string_buffer(256)
        n = self._lib.dart_debug_lm_head_key(self._h, rows, int(multi_row), buf, 256)
        if n < 0:
            raise RuntimeError("dart_debug_lm_head_key failed")
        return buf.value.decode()

    def debug_read(self, name: str, rows: int, cols: int) -> np.ndarray:
        buf = np.empty(16 * cols, dtype=np.float32)
        n = self._lib.dart_debug_read(self._h, name.encode(), buf.ctypes.data, buf.size)
        if n < 0:
            raise RuntimeError(f"dart_debug_read({name}) failed")
        return buf[: rows * cols].reshape(rows, cols).copy()


def debug_stream_read(buf, workgroups: int = 2048, stream=None, non_temporal: bool = True):
    """dart_debug_stream_read over a CUDA tensor (diagnostic: the box's streaming-read rate)."""
    lib = load_library()
    _check(lib.dart_debug_stream_read(buf.data_ptr(), buf.numel() * buf.element_size(), workgroups,
                                      int(non_temporal), None, _stream_ptr(stream)), "dart_debug_stream_read")


def topk_static(logits, k: int, eps: float = 1e-9, stream=None, out=None):
    """dart_topk_static: dart_topk on the library's built-in workspace (no context, no allocation
    inside the call; pass `out` = (ids, scores) to keep the caller side allocation-free too)."""
    torch = _torch()
    lib = load_library()
    rows, vocab = logits.shape
    if out is None:
        out = (torch.empty((rows, k), dtype=torch.int32, device=logits.device),
               torch.empty((rows, k), dtype=torch.float32, device=logits.device))
    ids, scores = out
    _check(lib.dart_topk_static(logits.data_ptr(), rows, vocab, k, eps, ids.data_ptr(),
                                scores.data_ptr(), _stream_ptr(stream)), "dart_topk_static")
    return ids, scores


def tree_verify_greedy(tokens, parents, n_nodes, ctx_len=None, target_next=None, path_cap: int = 17,
                       stream=None):
    """dart_tree_verify_greedy on CUDA int32 tensors [batch][budget] (n_nodes, ctx_len [batch]).
    Returns (position_ids, accept_path, n_accepted, next_token); the last three are None when
    target_next is None."""
    torch = _torch()
    lib = load_library()
    B, budget = tokens.shape
    dev = tokens.device
    pos = torch.empty((B, budget), dtype=torch.int32, device=dev)
    path = n_acc = nxt = None
    if target_next is not None:
        path = torch.empty((B, path_cap), dtype=torch.int32, device=dev)
        n_acc = torch.empty((B,), dtype=torch.int32, device=dev)
        nxt = torch.empty((B,), dtype=torch.int32, device=dev)
    ptr = lambda t: None if t is None else t.data_ptr()
    _check(lib.dart_tree_verify_greedy(B, tokens.data_ptr(), parents.data_ptr(), n_nodes.data_ptr(),
                                       budget, ptr(ctx_len), pos.data_ptr(), ptr(target_next),
                                       path_cap, ptr(path), ptr(n_acc), ptr(nxt),
                                       _stream_ptr(stream)), "dart_tree_verify_greedy")
    return pos, path, n_acc, nxt


class NgramTable:
    """dart_ngram: device hash table context -> successors, built from raw counts."""

    def __init__(self, n_gram: int, keys, succ_ids, succ_counts, eps: float = 1e-9):
        lib = load_library()
        keys = np.ascontiguousarray(keys, dtype=np.int32)
        succ_ids = np.ascontiguousarray(succ_ids, dtype=np.int32)
        succ_counts = np.ascontiguousarray(succ_counts, dtype=np.int32)
        n_keys = keys.shape[0]
        S = succ_ids.shape[1] if succ_ids.ndim == 2 else 1
        self.n_gram = n_gram
        handle = C.c_void_p()
        _check(lib.dart_ngram_create(n_gram, n_keys, S, keys.ctypes.data, succ_ids.ctypes.data,
                                     succ_counts.ctypes.data, eps, C.byref(handle)),
               "dart_ngram_create")
        self._h, self._lib = handle, lib

    def set_backoff(self, keys, succ_ids, succ_counts, alpha: float):
        """dart_ngram_set_backoff: attach a bigram table (keys [n][1]) consulted for trigram
        contexts this table lacks, with discount alpha."""
        keys = np.ascontiguousarray(keys, dtype=np.int32)
        succ_ids = np.ascontiguousarray(succ_ids, dtype=np.int32)
        succ_counts = np.ascontiguousarray(succ_counts, dtype=np.int32)
        _check(self._lib.dart_ngram_set_backoff(self._h, keys.shape[0], keys.ctypes.data,
                                                succ_ids.ctypes.data, succ_counts.ctypes.data, alpha),
               "dart_ngram_set_backoff")

    def close(self):
        if getattr(self, "_h", None):
            self._lib.dart_ngram_destroy(self._h)
            self._h = None

    __del__ = close

    def tree_prune(self, ids, scores, ctx_tail, params: PruneParams, stream=None, out=None):
        """dart_tree_prune: ids/scores CUDA [batch][K][k] (or [K][k]); ctx_tail [batch][N-1].

        Returns tokens [batch][budget], parents [batch][budget], mask [batch][budget][budget],
        n_nodes [batch] (CUDA tensors; the batch axis is dropped for 2-D inputs).  `out` may
        carry preallocated (tokens, parents, mask, n_nodes) tensors of the batched shapes."""
        torch = _torch()
        squeeze = ids.dim() == 2
        if squeeze:
            ids, scores, ctx_tail = ids[None], scores[None], ctx_tail[None]
        B, K, k = ids.shape
        if k != params.k or scores.shape != ids.shape:
            raise ValueError("ids/scores must be [batch][K][params.k]")
        ids = ids.contiguous()
        scores = scores.contiguous()
        ctx_tail = ctx_tail.contiguous()
        dev = ids.device
        if out is None:
            tokens = torch.empty((B, params.budget), dtype=torch.int32, device=dev)
            parents = torch.empty((B, params.budget), dtype=torch.int32, device=dev)
            mask = torch.empty((B, params.budget, params.budget), dtype=torch.uint8, device=dev)
            n_nodes = torch.empty((B,), dtype=torch.int32, device=dev)
        else:
            tokens, parents, mask, n_nodes = out
        p = _PruneParams(params.k, params.beam_w, params.budget, params.w_ng, params.logit_decay,
                         params.level_pow)
        _check(self._lib.dart_tree_prune(B, ids.data_ptr(), scores.data_ptr(), K,
                                         ctx_tail.data_ptr(), self._h, C.byref(p),
                                         tokens.data_ptr(), parents.data_ptr(), mask.data_ptr(),
                                         n_nodes.data_ptr(), _stream_ptr(stream)),
               "dart_tree_prune")
        if squeeze:
            return tokens[0], parents[0], mask[0], n_nodes[0]
        return tokens, parents, mask, n_nodes
