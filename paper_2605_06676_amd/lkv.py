"""Thin Python binding over the C ABI of include/lkv.h (ctypes).

Argument marshalling only: every step of the path runs in the HIP kernels of
the shared library.  torch tensors supply device memory and the stream.  There
is no fallback: if the library has not been built, or no GPU is present, the
calls raise.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("LKV_LIBRARY", os.path.join(_HERE, "liblkv.so"))   # LKV_LIBRARY: load another build of the library

LKV_OK = 0
SCORER_LINEAR, SCORER_MLP = 0, 1
ACT_SILU, ACT_GELU_ERF = 0, 1
POOL_MAX, POOL_AVG = 0, 1
_STATUS = {0: "LKV_OK", 1: "LKV_ERR_INVALID_ARG", 2: "LKV_ERR_UNSUPPORTED", 3: "LKV_ERR_WORKSPACE", 4: "LKV_ERR_HIP"}

EXPORTS = ("lkv_create", "lkv_destroy", "lkv_last_error", "lkv_version", "lkv_score",
           "lkv_score_window_workspace_bytes", "lkv_score_window", "lkv_select",
           "lkv_counts_bytes", "lkv_counts_bytes_split", "lkv_clear_counts", "lkv_score_counted", "lkv_select_counted",
           "lkv_compact", "lkv_decode_workspace_bytes", "lkv_decode_attn", "lkv_decode_attn_static", "lkv_soft_topk_max_n",
           "lkv_soft_topk", "lkv_soft_topk_backward", "lkv_soft_topk_batched", "lkv_soft_topk_backward_batched",
           "lkv_head_budgets", "lkv_plan_offsets", "lkv_evict_layer", "lkv_compact_grow",
           "lkv_append", "lkv_decode_attn_grown", "lkv_reevict", "lkv_masked_decode_workspace_bytes",
           "lkv_masked_decode_attn", "lkv_masked_attn_forward",
           "lkv_masked_attn_backward_workspace_bytes", "lkv_masked_attn_backward")


class LkvError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_STATUS.get(status, status)}: {message}")
        self.status = status


class _Cache(C.Structure):
    _fields_ = [("n_seq", C.c_int32), ("n_layers", C.c_int32), ("n_kv_heads", C.c_int32),
                ("n_q_heads", C.c_int32), ("head_dim", C.c_int32),
                ("seq_len", C.POINTER(C.c_int32)), ("k", C.POINTER(C.c_void_p)), ("v", C.POINTER(C.c_void_p))]


class _Scorer(C.Structure):
    _fields_ = [("kind", C.c_int32), ("act", C.c_int32), ("hidden", C.c_int32), ("per_head", C.c_int32),
                ("w1", C.c_void_p), ("b1", C.c_void_p), ("w2", C.c_void_p), ("b2", C.c_void_p)]


class _HeadPredictor(C.Structure):
    _fields_ = [("d_e", C.c_int32), ("hidden", C.c_int32), ("w1", C.c_void_p), ("b1", C.c_void_p),
                ("w2", C.c_void_p), ("b2", C.c_void_p)]


_lib = None


def load_library() -> C.CDLL:
    """Load liblkv.so (built by paper_2605_06676_amd/build.py); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} is missing: build it with `python -m paper_2605_06676_amd.build`")
    lib = C.CDLL(LIB_PATH)
    lib.lkv_create.argtypes = [C.POINTER(C.c_void_p), C.c_int]
    lib.lkv_create.restype = C.c_int
    lib.lkv_destroy.argtypes = [C.c_void_p]
    lib.lkv_destroy.restype = None
    lib.lkv_last_error.argtypes = [C.c_void_p]
    lib.lkv_last_error.restype = C.c_char_p
    lib.lkv_version.argtypes = []
    lib.lkv_version.restype = C.c_char_p
    lib.lkv_score.argtypes = [C.c_void_p, C.POINTER(_Cache), C.POINTER(_Scorer), C.POINTER(C.c_void_p), C.c_void_p]
    lib.lkv_score.restype = C.c_int
    lib.lkv_score_window_workspace_bytes.argtypes = [C.POINTER(_Cache)]
    lib.lkv_score_window_workspace_bytes.restype = C.c_size_t
    lib.lkv_score_window.argtypes = [C.c_void_p, C.POINTER(_Cache), C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_int32,
                                     C.c_int32, C.c_int32, C.c_float, C.POINTER(C.c_void_p), C.c_void_p, C.c_size_t,
                                     C.c_void_p]
    lib.lkv_score_window.restype = C.c_int
    lib.lkv_select.argtypes = [C.c_void_p, C.POINTER(_Cache), C.POINTER(C.c_void_p), C.POINTER(C.c_int32),
                               C.c_void_p, C.c_void_p, C.c_void_p]
    lib.lkv_select.restype = C.c_int
    lib.lkv_counts_bytes.argtypes = [C.c_int64]
    lib.lkv_counts_bytes.restype = C.c_size_t
    lib.lkv_counts_bytes_split.argtypes = [C.c_int64, C.c_int32]
    lib.lkv_counts_bytes_split.restype = C.c_size_t
    lib.lkv_clear_counts.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
    lib.lkv_clear_counts.restype = C.c_int
    lib.lkv_score_counted.argtypes = [C.c_void_p, C.POINTER(_Cache), C.POINTER(_Scorer), C.POINTER(C.c_void_p), C.c_void_p,
                                      C.c_void_p]
    lib.lkv_score_counted.restype = C.c_int
    lib.lkv_select_counted.argtypes = [C.c_void_p, C.POINTER(_Cache), C.POINTER(C.c_void_p), C.POINTER(C.c_int32),
                                       C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.lkv_select_counted.restype = C.c_int
    lib.lkv_compact.argtypes = [C.c_void_p, C.POINTER(_Cache), C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p,
                                C.c_void_p, C.c_void_p]
    lib.lkv_compact.restype = C.c_int
    lib.lkv_decode_workspace_bytes.argtypes = [C.c_int32, C.c_int64, C.c_int32, C.c_int32]
    lib.lkv_decode_workspace_bytes.restype = C.c_size_t
    lib.lkv_decode_attn.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                    C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_float, C.c_void_p,
                                    C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.lkv_decode_attn.restype = C.c_int
    lib.lkv_decode_attn_static.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                           C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_float, C.c_void_p,
                                           C.c_void_p, C.c_void_p]
    lib.lkv_decode_attn_static.restype = C.c_int
    lib.lkv_plan_offsets.argtypes = [C.c_void_p, C.c_int64, C.POINTER(C.c_int32), C.c_void_p, C.POINTER(C.c_int64),
                                     C.c_void_p]
    lib.lkv_plan_offsets.restype = C.c_int
    lib.lkv_evict_layer.argtypes = [C.c_void_p, C.POINTER(_Cache), C.c_int32, C.c_int32, C.POINTER(_Scorer),
                                    C.POINTER(C.c_int32), C.c_void_p, C.POINTER(C.c_void_p), C.c_void_p, C.c_void_p,
                                    C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.lkv_evict_layer.restype = C.c_int
    lib.lkv_compact_grow.argtypes = [C.c_void_p, C.POINTER(_Cache), C.POINTER(C.c_void_p), C.c_void_p, C.c_void_p,
                                     C.c_int64, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_void_p]
    lib.lkv_compact_grow.restype = C.c_int
    lib.lkv_append.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.POINTER(_Scorer), C.c_void_p,
                               C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                               C.c_void_p]
    lib.lkv_append.restype = C.c_int
    lib.lkv_decode_attn_grown.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                          C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_float,
                                          C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.lkv_decode_attn_grown.restype = C.c_int
    lib.lkv_reevict.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.c_int32, C.c_void_p,
                                C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                C.POINTER(C.c_int64), C.c_void_p]
    lib.lkv_reevict.restype = C.c_int
    lib.lkv_masked_decode_workspace_bytes.argtypes = [C.POINTER(_Cache)]
    lib.lkv_masked_decode_workspace_bytes.restype = C.c_size_t
    lib.lkv_masked_decode_attn.argtypes = [C.c_void_p, C.POINTER(_Cache), C.c_void_p, C.POINTER(C.c_void_p), C.c_float,
                                           C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.lkv_masked_decode_attn.restype = C.c_int
    lib.lkv_masked_attn_forward.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                            C.c_void_p, C.c_void_p, C.c_void_p, C.c_float, C.c_void_p, C.c_void_p,
                                            C.c_void_p]
    lib.lkv_masked_attn_forward.restype = C.c_int
    lib.lkv_masked_attn_backward_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32]
    lib.lkv_masked_attn_backward_workspace_bytes.restype = C.c_size_t
    lib.lkv_masked_attn_backward.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32] + [C.c_void_p] * 7 + [
        C.c_float] + [C.c_void_p] * 5 + [C.c_size_t, C.c_void_p]
    lib.lkv_masked_attn_backward.restype = C.c_int
    lib.lkv_soft_topk_max_n.argtypes = [C.c_int32]
    lib.lkv_soft_topk_max_n.restype = C.c_int32
    lib.lkv_soft_topk.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_double, C.c_double, C.c_void_p,
                                  C.c_void_p, C.c_void_p]
    lib.lkv_soft_topk.restype = C.c_int
    lib.lkv_soft_topk_backward.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_double, C.c_void_p,
                                           C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.lkv_soft_topk_backward.restype = C.c_int
    lib.lkv_soft_topk_batched.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_double,
                                          C.c_void_p, C.c_void_p, C.c_void_p]
    lib.lkv_soft_topk_batched.restype = C.c_int
    lib.lkv_soft_topk_backward_batched.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_double,
                                                   C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.lkv_soft_topk_backward_batched.restype = C.c_int
    lib.lkv_head_budgets.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(_HeadPredictor), C.c_int32, C.c_double,
                                     C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.lkv_head_budgets.restype = C.c_int
    _lib = lib
    return lib


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _stream_ptr(stream) -> Optional[int]:
    import torch

    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


class Cache:
    """Host-side description of a prefilled cache: lists of per-sequence K and V tensors,
    each bf16 [L, H, T_s, 128] and contiguous on the GPU."""

    def __init__(self, k: Sequence, v: Sequence, n_q_heads: int):
        import torch

        assert len(k) == len(v) and len(k) >= 1
        L, H, _, d = k[0].shape
        for a, b in zip(k, v):
            assert a.dtype == torch.bfloat16 and b.dtype == torch.bfloat16
            assert a.is_cuda and b.is_cuda and a.is_contiguous() and b.is_contiguous()
            assert a.shape == b.shape and a.shape[0] == L and a.shape[1] == H and a.shape[3] == d
        self.k, self.v = list(k), list(v)
        self.n_seq, self.L, self.H, self.Hq, self.d = len(k), L, H, n_q_heads, d
        self.seq_len = [int(a.shape[2]) for a in k]
        self._lens = (C.c_int32 * self.n_seq)(*self.seq_len)
        self._kp = (C.c_void_p * self.n_seq)(*[a.data_ptr() for a in k])
        self._vp = (C.c_void_p * self.n_seq)(*[a.data_ptr() for a in v])
        self.c = _Cache(self.n_seq, L, H, n_q_heads, d, self._lens, self._kp, self._vp)

    @property
    def n_segments(self) -> int:
        return self.n_seq * self.L * self.H


class Context:
    def __init__(self, device: int = 0):
        self.lib = load_library()
        self.h = C.c_void_p()
        st = self.lib.lkv_create(C.byref(self.h), device)
        if st != LKV_OK:
            raise LkvError(st, "lkv_create failed (is a GPU present?)")

    def close(self):
        if self.h:
            self.lib.lkv_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int):
        if st != LKV_OK:
            raise LkvError(st, self.lib.lkv_last_error(self.h).decode())


def _scorer_struct(scorer: dict) -> _Scorer:
    kind = SCORER_LINEAR if scorer["kind"] == "linear" else SCORER_MLP
    act = ACT_SILU if scorer.get("act", "silu") == "silu" else ACT_GELU_ERF
    return _Scorer(kind, act, int(scorer.get("hidden", 0)), int(bool(scorer.get("per_head", False))),
                   _ptr(scorer["w1"]), _ptr(scorer["b1"]), _ptr(scorer.get("w2")), _ptr(scorer.get("b2")))


def lkv_score(ctx: Context, cache: Cache, scorer: dict, scores: Sequence, stream=None) -> None:
    """scorer: dict(kind, act, hidden, per_head, w1, b1, w2, b2) of GPU tensors (w1 bf16, others fp32).
    scores: per-sequence fp32 [L, H, T_s] GPU tensors, written in place."""
    sc = _scorer_struct(scorer)
    sp = (C.c_void_p * cache.n_seq)(*[s.data_ptr() for s in scores])
    ctx._check(ctx.lib.lkv_score(ctx.h, C.byref(cache.c), C.byref(sc), sp, _stream_ptr(stream)))


def lkv_score_window_workspace_bytes(cache: Cache) -> int:
    return int(load_library().lkv_score_window_workspace_bytes(C.byref(cache.c)))


def lkv_score_window(ctx: Context, cache: Cache, q_win: Sequence, window: int, pool_width: int, pool_kind: int,
                     scale: float, scores: Sequence, workspace, stream=None, lse_win: Optional[Sequence] = None) -> None:
    """q_win: per-sequence bf16 [L, Hq, window, 128] GPU tensors (the queries of the last `window` positions);
    scores: per-sequence fp32 [L, H, T_s] GPU tensors, written in place; lse_win: None, or per-sequence fp32
    [L, Hq, window] GPU tensors with the log-normalisers of those queries (then the keys are read once)."""
    import torch

    assert all(q.dtype == torch.bfloat16 and q.is_contiguous() for q in q_win)
    assert all(s.dtype == torch.float32 and s.is_contiguous() for s in scores)
    qp = (C.c_void_p * cache.n_seq)(*[q.data_ptr() for q in q_win])
    sp = (C.c_void_p * cache.n_seq)(*[s.data_ptr() for s in scores])
    lp = None
    if lse_win is not None:
        assert all(t.dtype == torch.float32 and t.is_contiguous() for t in lse_win)
        lp = (C.c_void_p * cache.n_seq)(*[t.data_ptr() for t in lse_win])
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    ctx._check(ctx.lib.lkv_score_window(ctx.h, C.byref(cache.c), qp, lp, int(window), int(pool_width), int(pool_kind),
                                        float(scale), sp, _ptr(workspace), ws_bytes, _stream_ptr(stream)))


def lkv_select(ctx: Context, cache: Cache, scores: Sequence, budgets, idx, offsets, stream=None) -> None:
    """budgets: host int32 array [n_seq * L * H], or None when `offsets` already holds what lkv_plan_offsets wrote for
    them; idx (int32 [sum b]) and offsets (int32 [n_seg + 1]) GPU tensors."""
    import numpy as np

    bp = None
    if budgets is not None:
        b = np.ascontiguousarray(np.asarray(budgets, dtype=np.int32).reshape(-1))
        assert b.size == cache.n_segments
        bp = b.ctypes.data_as(C.POINTER(C.c_int32))
    sp = (C.c_void_p * cache.n_seq)(*[s.data_ptr() for s in scores])
    ctx._check(ctx.lib.lkv_select(ctx.h, C.byref(cache.c), sp, bp, _ptr(idx), _ptr(offsets), _stream_ptr(stream)))


def lkv_counts_bytes(n_segments: int) -> int:
    return int(load_library().lkv_counts_bytes(int(n_segments)))


def lkv_counts_bytes_split(n_segments: int, max_seq_len: int) -> int:
    return int(load_library().lkv_counts_bytes_split(int(n_segments), int(max_seq_len)))


def lkv_clear_counts(ctx: Context, counts, n_segments: int, stream=None) -> None:
    """counts: GPU uint8/int32 buffer of lkv_counts_bytes(n_segments) bytes; zeroed by a fill kernel."""
    assert counts.numel() * counts.element_size() >= lkv_counts_bytes(n_segments)
    ctx._check(ctx.lib.lkv_clear_counts(ctx.h, _ptr(counts), int(n_segments), _stream_ptr(stream)))


def lkv_score_counted(ctx: Context, cache: Cache, scorer: dict, scores: Sequence, counts, stream=None) -> None:
    """lkv_score that also counts the first-level top-k digits per segment into `counts` (zero on entry)."""
    assert counts.numel() * counts.element_size() >= lkv_counts_bytes(cache.n_segments)
    sc = _scorer_struct(scorer)
    sp = (C.c_void_p * cache.n_seq)(*[s.data_ptr() for s in scores])
    ctx._check(ctx.lib.lkv_score_counted(ctx.h, C.byref(cache.c), C.byref(sc), sp, _ptr(counts), _stream_ptr(stream)))


def lkv_select_counted(ctx: Context, cache: Cache, scores: Sequence, budgets, counts, idx, offsets, stream=None) -> None:
    """lkv_select that starts from the counts lkv_score_counted left (and zeroes them again)."""
    import numpy as np

    assert counts.numel() * counts.element_size() >= lkv_counts_bytes(cache.n_segments)
    bp = None
    if budgets is not None:
        b = np.ascontiguousarray(np.asarray(budgets, dtype=np.int32).reshape(-1))
        assert b.size == cache.n_segments
        bp = b.ctypes.data_as(C.POINTER(C.c_int32))
    sp = (C.c_void_p * cache.n_seq)(*[s.data_ptr() for s in scores])
    ctx._check(ctx.lib.lkv_select_counted(ctx.h, C.byref(cache.c), sp, bp, _ptr(counts), _ptr(idx), _ptr(offsets),
                                          _stream_ptr(stream)))


def lkv_compact(ctx: Context, cache: Cache, idx, offsets, total_kept: int, kp, vp, stream=None) -> None:
    ctx._check(ctx.lib.lkv_compact(ctx.h, C.byref(cache.c), _ptr(idx), _ptr(offsets), int(total_kept),
                                   _ptr(kp), _ptr(vp), _stream_ptr(stream)))


def lkv_decode_workspace_bytes(n_segments: int, total_kept: int, n_q_heads: int, n_kv_heads: int) -> int:
    return int(load_library().lkv_decode_workspace_bytes(n_segments, int(total_kept), n_q_heads, n_kv_heads))


def lkv_decode_attn(ctx: Context, n_seq: int, L: int, H: int, Hq: int, d: int, q, kp, vp, offsets,
                    total_kept: int, scale: float, out, lse, workspace, stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    ctx._check(ctx.lib.lkv_decode_attn(ctx.h, n_seq, L, H, Hq, d, _ptr(q), _ptr(kp), _ptr(vp), _ptr(offsets),
                                       int(total_kept), float(scale), _ptr(out), _ptr(lse), _ptr(workspace),
                                       ws_bytes, _stream_ptr(stream)))


DECODE_STATIC_SCRATCH_BYTES = 16 << 20


def lkv_decode_attn_static(ctx: Context, n_seq: int, L: int, H: int, Hq: int, d: int, q, kp, vp, offsets,
                           total_kept: int, scale: float, out, lse, stream=None) -> None:
    """lkv_decode_attn without a workspace argument: the partials go to the library's static device array."""
    ctx._check(ctx.lib.lkv_decode_attn_static(ctx.h, n_seq, L, H, Hq, d, _ptr(q), _ptr(kp), _ptr(vp), _ptr(offsets),
                                              int(total_kept), float(scale), _ptr(out), _ptr(lse), _stream_ptr(stream)))


def lkv_soft_topk_max_n(x_is_f64: bool) -> int:
    return int(load_library().lkv_soft_topk_max_n(1 if x_is_f64 else 0))


def lkv_soft_topk(ctx: Context, x, k: float, tau: float, y, info=None, stream=None) -> None:
    """x: GPU fp32 or fp64 [n]; y: GPU fp64 [n]; info: GPU fp64 [2] or None."""
    import torch

    assert x.dtype in (torch.float32, torch.float64) and x.is_contiguous()
    assert y.dtype == torch.float64 and y.numel() == x.numel() and y.is_contiguous()
    assert info is None or (info.dtype == torch.float64 and info.numel() >= 2)
    ctx._check(ctx.lib.lkv_soft_topk(ctx.h, _ptr(x), 1 if x.dtype == torch.float64 else 0, int(x.numel()), float(k),
                                     float(tau), _ptr(y), _ptr(info), _stream_ptr(stream)))


def lkv_soft_topk_backward(ctx: Context, x, tau: float, info, g, dx, dk=None, stream=None) -> None:
    """x: the forward call's input; info: GPU fp64 [2] as that call wrote it; g, dx: GPU fp64 [n]; dk: GPU fp64 [1] or None."""
    import torch

    assert x.dtype in (torch.float32, torch.float64) and x.is_contiguous()
    assert info.dtype == torch.float64 and info.numel() >= 2
    assert all(t.dtype == torch.float64 and t.numel() == x.numel() and t.is_contiguous() for t in (g, dx))
    assert dk is None or (dk.dtype == torch.float64 and dk.numel() >= 1)
    ctx._check(ctx.lib.lkv_soft_topk_backward(ctx.h, _ptr(x), 1 if x.dtype == torch.float64 else 0, int(x.numel()),
                                              float(tau), _ptr(info), _ptr(g), _ptr(dx), _ptr(dk), _stream_ptr(stream)))


def lkv_soft_topk_batched(ctx: Context, x, k, tau: float, y, info=None, stream=None) -> None:
    """x: GPU fp32 or fp64 [n_vec, n]; k: GPU fp64 [n_vec]; y: GPU fp64 [n_vec, n]; info: GPU fp64 [n_vec, 2] or None."""
    import torch

    assert x.dim() == 2 and x.dtype in (torch.float32, torch.float64) and x.is_contiguous()
    assert k.dtype == torch.float64 and k.numel() == x.shape[0] and k.is_contiguous()
    assert y.dtype == torch.float64 and y.shape == x.shape and y.is_contiguous()
    assert info is None or (info.dtype == torch.float64 and info.numel() == 2 * x.shape[0] and info.is_contiguous())
    ctx._check(ctx.lib.lkv_soft_topk_batched(ctx.h, _ptr(x), 1 if x.dtype == torch.float64 else 0, int(x.shape[0]),
                                             int(x.shape[1]), _ptr(k), float(tau), _ptr(y), _ptr(info), _stream_ptr(stream)))


def lkv_soft_topk_backward_batched(ctx: Context, x, tau: float, info, g, dx, dk=None, stream=None) -> None:
    """x [n_vec, n] as given to the forward call; info: GPU fp64 [n_vec, 2]; g, dx: GPU fp64 [n_vec, n]; dk: GPU fp64 [n_vec] or None."""
    import torch

    assert x.dim() == 2 and x.dtype in (torch.float32, torch.float64) and x.is_contiguous()
    assert info.dtype == torch.float64 and info.numel() == 2 * x.shape[0] and info.is_contiguous()
    assert all(t.dtype == torch.float64 and t.shape == x.shape and t.is_contiguous() for t in (g, dx))
    assert dk is None or (dk.dtype == torch.float64 and dk.numel() == x.shape[0] and dk.is_contiguous())
    ctx._check(ctx.lib.lkv_soft_topk_backward_batched(ctx.h, _ptr(x), 1 if x.dtype == torch.float64 else 0, int(x.shape[0]),
                                                      int(x.shape[1]), float(tau), _ptr(info), _ptr(g), _ptr(dx), _ptr(dk),
                                                      _stream_ptr(stream)))


def lkv_head_budgets(ctx: Context, emb, predictor: dict, R: float, t: int, r, b=None, stream=None) -> None:
    """emb: GPU fp32 [n_heads, d_e]; predictor: dict of GPU fp32 tensors w1 [hidden, d_e], b1, w2 and
    b2 ([1]) or None; r: GPU fp64 [n_heads]; b: GPU int32 [n_heads] or None."""
    import torch

    n_heads, d_e = emb.shape
    hidden = predictor["w1"].shape[0]
    for name in ("w1", "b1", "w2"):
        assert predictor[name].dtype == torch.float32 and predictor[name].is_contiguous()
    assert emb.dtype == torch.float32 and emb.is_contiguous() and predictor["w1"].shape[1] == d_e
    assert r.dtype == torch.float64 and r.numel() == n_heads
    assert b is None or (b.dtype == torch.int32 and b.numel() == n_heads)
    p = _HeadPredictor(d_e, hidden, _ptr(predictor["w1"]), _ptr(predictor["b1"]), _ptr(predictor["w2"]),
                       _ptr(predictor.get("b2")))
    ctx._check(ctx.lib.lkv_head_budgets(ctx.h, _ptr(emb), C.byref(p), n_heads, float(R), int(t), _ptr(r), _ptr(b),
                                        _stream_ptr(stream)))


def lkv_plan_offsets(ctx: Context, budgets, offsets, stream=None) -> int:
    """budgets: host int32 [n_segments]; offsets: GPU int32 [n_segments + 1].  Returns the total kept."""
    import numpy as np

    b = np.ascontiguousarray(np.asarray(budgets, dtype=np.int32).reshape(-1))
    assert offsets.numel() >= b.size + 1
    total = C.c_int64(0)
    ctx._check(ctx.lib.lkv_plan_offsets(ctx.h, b.size, b.ctypes.data_as(C.POINTER(C.c_int32)), _ptr(offsets),
                                        C.byref(total), _stream_ptr(stream)))
    return int(total.value)


def lkv_evict_layer(ctx: Context, layer: Cache, layer_index: int, n_layers: int, scorer: dict, budgets, offsets,
                    scores: Sequence, idx, kp, vp, stream=None, counts=None) -> None:
    """layer: a Cache built from per-sequence tensors [m, H, T_s, 128] of m consecutive layers starting at
    layer_index; budgets: host int32 [n_seq * n_layers * H]; scores: per-sequence GPU fp32 [m, H, T_s] scratch."""
    import numpy as np

    b = np.ascontiguousarray(np.asarray(budgets, dtype=np.int32).reshape(-1))
    assert b.size == layer.n_seq * n_layers * layer.H
    sc = None if scorer is None else C.byref(_scorer_struct(scorer))     # None: `scores` is an input
    sp = (C.c_void_p * layer.n_seq)(*[s.data_ptr() for s in scores])
    ctx._check(ctx.lib.lkv_evict_layer(ctx.h, C.byref(layer.c), layer_index, n_layers, sc,
                                       b.ctypes.data_as(C.POINTER(C.c_int32)), _ptr(offsets), sp, _ptr(idx), _ptr(kp),
                                       _ptr(vp), _ptr(counts), 0 if counts is None else counts.numel() * counts.element_size(),
                                       _stream_ptr(stream)))


def lkv_compact_grow(ctx: Context, cache: Cache, scores: Sequence, idx, offsets, total_kept: int, slack: int, kp, vp,
                     up, cap_offsets, lengths, stream=None) -> None:
    """kp, vp: bf16 [total_kept + n_segments * slack, 128]; up: fp32 of as many rows; cap_offsets int32
    [n_segments + 1] and lengths int32 [n_segments] are written."""
    sp = (C.c_void_p * cache.n_seq)(*[s.data_ptr() for s in scores])
    ctx._check(ctx.lib.lkv_compact_grow(ctx.h, C.byref(cache.c), sp, _ptr(idx), _ptr(offsets), int(total_kept),
                                        int(slack), _ptr(kp), _ptr(vp), _ptr(up), _ptr(cap_offsets), _ptr(lengths),
                                        _stream_ptr(stream)))


def lkv_append(ctx: Context, n_seq: int, L: int, H: int, d: int, scorer: dict, k_new, v_new, kp, vp, up, cap_offsets,
               lengths, overflow=None, stream=None) -> None:
    """k_new, v_new: bf16 [n_seq, L, H, 128]; overflow: int32 [1] GPU tensor or None."""
    sc = _scorer_struct(scorer)
    ctx._check(ctx.lib.lkv_append(ctx.h, n_seq, L, H, d, C.byref(sc), _ptr(k_new), _ptr(v_new), _ptr(kp), _ptr(vp),
                                  _ptr(up), _ptr(cap_offsets), _ptr(lengths), _ptr(overflow), _stream_ptr(stream)))


def lkv_decode_attn_grown(ctx: Context, n_seq: int, L: int, H: int, Hq: int, d: int, q, kp, vp, cap_offsets, lengths,
                          total_rows: int, scale: float, out, lse, workspace, stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    ctx._check(ctx.lib.lkv_decode_attn_grown(ctx.h, n_seq, L, H, Hq, d, _ptr(q), _ptr(kp), _ptr(vp), _ptr(cap_offsets),
                                             _ptr(lengths), int(total_rows), float(scale), _ptr(out), _ptr(lse),
                                             _ptr(workspace), ws_bytes, _stream_ptr(stream)))


def lkv_reevict(ctx: Context, d: int, kp, vp, up, cap_offsets, lengths, lengths_host, new_budgets, slack: int, idx,
                offsets, kp_new, vp_new, up_new, cap_offsets_new, lengths_new, stream=None) -> int:
    """Shrinks a cache with slack to new_budgets (host int32 [n_segments]) and returns the rows kept."""
    import numpy as np

    lh = np.ascontiguousarray(np.asarray(lengths_host, dtype=np.int32).reshape(-1))
    nb = np.ascontiguousarray(np.asarray(new_budgets, dtype=np.int32).reshape(-1))
    assert lh.size == nb.size
    total = C.c_int64(0)
    ctx._check(ctx.lib.lkv_reevict(ctx.h, lh.size, d, _ptr(kp), _ptr(vp), _ptr(up), _ptr(cap_offsets), _ptr(lengths),
                                   lh.ctypes.data_as(C.POINTER(C.c_int32)), nb.ctypes.data_as(C.POINTER(C.c_int32)),
                                   int(slack), _ptr(idx), _ptr(offsets), _ptr(kp_new), _ptr(vp_new), _ptr(up_new),
                                   _ptr(cap_offsets_new), _ptr(lengths_new), C.byref(total), _stream_ptr(stream)))
    return int(total.value)


def lkv_masked_decode_workspace_bytes(cache: Cache) -> int:
    return int(load_library().lkv_masked_decode_workspace_bytes(C.byref(cache.c)))


def lkv_masked_decode_attn(ctx: Context, cache: Cache, q, mask: Sequence, scale: float, out, lse, workspace,
                           stream=None) -> None:
    """mask: per-sequence GPU fp32 [L, H, T_s] with values in [0, 1]."""
    mp = (C.c_void_p * cache.n_seq)(*[m.data_ptr() for m in mask])
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    ctx._check(ctx.lib.lkv_masked_decode_attn(ctx.h, C.byref(cache.c), _ptr(q), mp, float(scale), _ptr(out), _ptr(lse),
                                              _ptr(workspace), ws_bytes, _stream_ptr(stream)))


def lkv_masked_attn_forward(ctx: Context, q, k, v, m, scale: float, o, lse, stream=None) -> None:
    """q: bf16 [Hq, T, 128]; k, v: bf16 [H, T, 128]; m: fp32 [H, T]; o: fp32 [Hq, T, 128]; lse: fp32 [Hq, T]."""
    import torch

    Hq, T, d = q.shape
    H = k.shape[0]
    # what the library cannot see from pointers: element types and contiguity (sizes and head counts are its to check)
    for t in (q, k, v):
        assert t.dtype == torch.bfloat16 and t.is_cuda and t.is_contiguous()
    for t in (m, o, lse):
        assert t is None or (t.dtype == torch.float32 and t.is_cuda and t.is_contiguous())
    ctx._check(ctx.lib.lkv_masked_attn_forward(ctx.h, Hq, H, T, d, _ptr(q), _ptr(k), _ptr(v), _ptr(m), float(scale),
                                               _ptr(o), _ptr(lse), _stream_ptr(stream)))


def lkv_masked_attn_backward_workspace_bytes(n_q_heads: int, n_kv_heads: int, seq_len: int) -> int:
    return int(load_library().lkv_masked_attn_backward_workspace_bytes(n_q_heads, n_kv_heads, seq_len))


def lkv_masked_attn_backward(ctx: Context, q, k, v, m, o, lse, d_o, scale: float, dq, dk, dv, dm, workspace,
                             stream=None) -> None:
    """q, d_o: bf16 [Hq, T, 128]; k, v: bf16 [H, T, 128]; m: fp32 [H, T]; o: fp32 [Hq, T, 128]; lse: fp32 [Hq, T];
    dq fp32 [Hq, T, 128]; dk, dv fp32 [H, T, 128]; dm fp32 [H, T]."""
    import torch

    Hq, T, d = q.shape
    H = k.shape[0]
    for t in (q, k, v, d_o):
        assert t.dtype == torch.bfloat16 and t.is_cuda and t.is_contiguous()
    for t in (m, o, lse, dq, dk, dv, dm):
        assert t is None or (t.dtype == torch.float32 and t.is_cuda and t.is_contiguous())
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    ctx._check(ctx.lib.lkv_masked_attn_backward(ctx.h, Hq, H, T, d, _ptr(q), _ptr(k), _ptr(v), _ptr(m), _ptr(o),
                                                _ptr(lse), _ptr(d_o), float(scale), _ptr(dq), _ptr(dk), _ptr(dv),
                                                _ptr(dm), _ptr(workspace), ws_bytes, _stream_ptr(stream)))
