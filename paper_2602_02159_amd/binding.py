"""ctypes binding of libfocus_hip.so: argument marshalling only.

Every function has the name of the C entry point it wraps (include/focus.h) minus the `focus_` prefix of
the status code: it takes torch CUDA tensors, passes their device pointers, sizes and strides through, and
raises FocusError on a non-zero status.  No step of the method runs in Python, and there is no fallback:
if the HIP library is not built, importing this module's `lib()` fails.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfocus_hip.so")

FOCUS_OK, FOCUS_EINVAL, FOCUS_EUNSUPPORTED, FOCUS_EWORKSPACE, FOCUS_ELAUNCH = 0, -1, -2, -3, -4
FN_BLOCK_SCORES, FN_FIND_SINKS, FN_SPARSE_ATTN, FN_SPARSE_LAYER, FN_PROBE_LAYER = 1, 2, 3, 4, 5

EXPORTS = ("focus_select_queries", "focus_expand_groups", "focus_block_means", "focus_block_scores", "focus_find_sinks", "focus_sparse_attn",
           "focus_sparse_layer", "focus_sparse_layer_static", "focus_block_partials", "focus_top_blocks", "focus_probe_layer", "focus_refresh_attn", "focus_cache_refresh",
           "focus_token_confidence", "focus_token_confidence_workspace", "focus_cache_update",
           "focus_workspace_bytes", "focus_helper_k", "focus_helper_n_keep", "focus_helper_n_sink", "focus_last_error",
           "focus_version")


class FocusError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"focus status {status}: {message}")
        self.status = status


class Shape(C.Structure):
    """Mirror of `focus_shape`."""
    _fields_ = [("n_heads", C.c_int32), ("head_dim", C.c_int32), ("n_ctx", C.c_int32), ("n_resp", C.c_int32),
                ("block", C.c_int32), ("n_gen", C.c_int32),
                ("q_stride_h", C.c_int64), ("q_stride_n", C.c_int64), ("k_stride_h", C.c_int64), ("k_stride_n", C.c_int64),
                ("v_stride_h", C.c_int64), ("v_stride_n", C.c_int64), ("o_stride_h", C.c_int64), ("o_stride_n", C.c_int64)]


_lib = None


def lib() -> C.CDLL:
    """The loaded library; raises if it has not been built (python -m paper_2602_02159_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is not built: run `python -m paper_2602_02159_amd.build`")
        L = C.CDLL(LIB_PATH)
        p, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
        sp = C.POINTER(Shape)
        L.focus_select_queries.argtypes = [p, p, i32, i32, i32, i32, i32, p, p, i32, p, p]
        L.focus_expand_groups.argtypes = [p, i32, p, i32, p, i32, i32, p, p, p, p]
        L.focus_block_means.argtypes = [p, sp, p, p]
        L.focus_block_scores.argtypes = [p, p, p, i32, p, p, sp, i32, p, p, p, sz, p]
        L.focus_find_sinks.argtypes = [p, p, p, i32, p, sp, i32, p, p, p, sz, p]
        L.focus_sparse_attn.argtypes = [p, p, p, i32, p, p, sp, p, i32, p, i32, p, p, p, sz, p]
        L.focus_sparse_layer.argtypes = [p, p, p, p, i32, i32, p, p, p, sp, i32, p, i32, p, p, p, p, p, sz, p]
        L.focus_sparse_layer_static.argtypes = [p, p, p, p, i32, i32, p, p, p, sp, i32, p, i32, p, p, p, p, p]
        L.focus_probe_layer.argtypes = [p, p, p, i32, p, p, sp, i32, p, p, p, p, p, sz, p]
        L.focus_refresh_attn.argtypes = [p, p, p, sp, p, p, p]
        L.focus_cache_refresh.argtypes = [p, p, sp, p, p, C.c_int64, C.c_int64, p, p]
        L.focus_token_confidence.argtypes = [p, C.c_int64, p, i32, i32, p, p, p, sz, p]
        L.focus_token_confidence_workspace.argtypes = [i32, i32]
        L.focus_token_confidence_workspace.restype = sz
        L.focus_cache_update.argtypes = [p, p, sp, p, p, C.c_int64, C.c_int64, p, p, i32, i32, p]
        L.focus_block_partials.argtypes = [p, p, p, i32, p, p, sp, p, p]
        L.focus_top_blocks.argtypes = [p, i32, p, i32, i32, i32, p, p, p]
        for name in ("focus_select_queries", "focus_expand_groups", "focus_block_means", "focus_block_scores", "focus_find_sinks",
                     "focus_sparse_attn", "focus_sparse_layer", "focus_sparse_layer_static", "focus_block_partials", "focus_top_blocks",
                     "focus_probe_layer", "focus_refresh_attn", "focus_token_confidence", "focus_cache_update", "focus_cache_refresh"):
            getattr(L, name).restype = C.c_int
        L.focus_workspace_bytes.argtypes = [i32, sp, i32, i32, i32]
        L.focus_workspace_bytes.restype = sz
        L.focus_helper_k.argtypes = [C.c_double, i32]
        L.focus_helper_k.restype = i32
        L.focus_helper_n_keep.argtypes = [C.c_double, i32]
        L.focus_helper_n_keep.restype = i32
        L.focus_helper_n_sink.argtypes = [C.c_double, i32]
        L.focus_helper_n_sink.restype = i32
        L.focus_last_error.restype = C.c_char_p
        L.focus_version.restype = C.c_char_p
        _lib = L
    return _lib


def last_error() -> str:
    return lib().focus_last_error().decode()


def _check(status: int) -> None:
    if status != FOCUS_OK:
        raise FocusError(status, last_error())


def _ptr(t) -> int | None:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _need(t: torch.Tensor, dtype, name: str) -> None:
    if not t.is_cuda or t.dtype != dtype:
        raise TypeError(f"{name}: expected a CUDA tensor of {dtype}, got {t.dtype} on {t.device}")


def make_shape(q: torch.Tensor, k: torch.Tensor | None, v: torch.Tensor | None, n_ctx: int, block: int,
               out: torch.Tensor | None = None) -> Shape:
    """focus_shape from [H, rows, d] tensors (any strides with a unit innermost stride)."""
    H, n_gen, d = q.shape
    s = Shape()
    s.n_heads, s.head_dim, s.n_gen, s.block, s.n_ctx = H, d, n_gen, block, n_ctx
    ref = k if k is not None else v
    s.n_resp = (ref.shape[1] - n_ctx) if ref is not None else 0
    for name, t in (("q", q), ("k", k), ("v", v), ("o", out)):
        if t is None:
            continue
        if t.stride(2) != 1:
            raise ValueError(f"{name}: innermost stride must be 1")
        setattr(s, f"{name}_stride_h", t.stride(0))
        setattr(s, f"{name}_stride_n", t.stride(1))
    return s


def workspace_bytes(fn: int, shape: Shape, max_active: int = 1, n_keep: int = 0, n_sink: int = 0) -> int:
    return int(lib().focus_workspace_bytes(fn, C.byref(shape), max_active, n_keep, n_sink))


def helper_k(rho: float, n_unmask: int) -> int:
    return int(lib().focus_helper_k(rho, n_unmask))


def helper_n_keep(alpha: float, n_blocks: int) -> int:
    return int(lib().focus_helper_n_keep(alpha, n_blocks))


def helper_n_sink(frac: float, n_ctx: int) -> int:
    return int(lib().focus_helper_n_sink(frac, n_ctx))


def select_queries(conf, masked, k: int, window: int, lo: int, hi: int, focus_idx, active_idx, counts) -> None:
    _need(conf, torch.float32, "conf")
    _check(lib().focus_select_queries(_ptr(conf), _ptr(masked), conf.numel(), k, window, lo, hi, _ptr(focus_idx),
                                      _ptr(active_idx), active_idx.numel(), _ptr(counts), _stream()))


def expand_groups(focus_idx, active_idx, counts, n_gen: int, group: int, focus_out, active_out, counts_out) -> None:
    """Index lists of select_queries -> lists of rows g * n_gen + i of the [H_kv, group * n_gen, d] view of Q."""
    _check(lib().focus_expand_groups(_ptr(focus_idx), focus_idx.numel(), _ptr(active_idx), active_idx.numel(), _ptr(counts),
                                     n_gen, group, _ptr(focus_out), _ptr(active_out), _ptr(counts_out), _stream()))


def block_means(k, shape: Shape, kbar) -> None:
    _need(k, torch.bfloat16, "K")
    _check(lib().focus_block_means(_ptr(k), C.byref(shape), _ptr(kbar), _stream()))


def block_scores(q, focus_idx, counts, k, kbar, shape: Shape, n_keep: int, scores, kept_blocks, workspace) -> None:
    _need(q, torch.bfloat16, "Q")
    _check(lib().focus_block_scores(_ptr(q), _ptr(focus_idx), _ptr(counts), focus_idx.numel(), _ptr(k), _ptr(kbar),
                                    C.byref(shape), n_keep, _ptr(scores), _ptr(kept_blocks), _ptr(workspace),
                                    0 if workspace is None else workspace.numel() * workspace.element_size(), _stream()))


def block_partials(q, focus_idx, counts, k, kbar, shape: Shape, partials) -> None:
    _need(q, torch.bfloat16, "Q")
    _need(partials, torch.float32, "partials")
    _check(lib().focus_block_partials(_ptr(q), _ptr(focus_idx), _ptr(counts), focus_idx.numel(), _ptr(k), _ptr(kbar),
                                      C.byref(shape), _ptr(partials), _stream()))


def top_blocks(partials, counts, n_focus_max: int, n_keep: int, scores, kept_blocks) -> None:
    _need(partials, torch.float32, "partials")
    n_parts, n_blocks = partials.shape
    _check(lib().focus_top_blocks(_ptr(partials), n_parts, _ptr(counts), n_focus_max, n_blocks, n_keep, _ptr(scores),
                                  _ptr(kept_blocks), _stream()))


def find_sinks(q, active_idx, counts, k, shape: Shape, n_sink: int, col_mass, sink_idx, workspace) -> None:
    _need(q, torch.bfloat16, "Q")
    _need(k, torch.bfloat16, "K")
    _check(lib().focus_find_sinks(_ptr(q), _ptr(active_idx), _ptr(counts), active_idx.numel(), _ptr(k), C.byref(shape),
                                  n_sink, _ptr(col_mass), _ptr(sink_idx), _ptr(workspace),
                                  0 if workspace is None else workspace.numel() * workspace.element_size(), _stream()))


def sparse_attn(q, active_idx, counts, k, v, shape: Shape, kept_blocks, n_keep: int, sink_idx, n_sink: int, out, lse,
                workspace) -> None:
    _need(q, torch.bfloat16, "Q")
    _need(k, torch.bfloat16, "K")
    _need(v, torch.bfloat16, "V")
    _need(out, torch.bfloat16, "out")
    _check(lib().focus_sparse_attn(_ptr(q), _ptr(active_idx), _ptr(counts), active_idx.numel(), _ptr(k), _ptr(v),
                                   C.byref(shape), _ptr(kept_blocks), n_keep, _ptr(sink_idx), n_sink, _ptr(out), _ptr(lse),
                                   _ptr(workspace),
                                   0 if workspace is None else workspace.numel() * workspace.element_size(), _stream()))


def probe_layer(q, active_idx, counts, k, v, shape: Shape, n_sink: int, out, lse, col_mass, sink_idx, workspace) -> None:
    _need(q, torch.bfloat16, "Q")
    _need(k, torch.bfloat16, "K")
    _need(v, torch.bfloat16, "V")
    _need(out, torch.bfloat16, "out")
    _check(lib().focus_probe_layer(_ptr(q), _ptr(active_idx), _ptr(counts), active_idx.numel(), _ptr(k), _ptr(v),
                                   C.byref(shape), n_sink, _ptr(out), _ptr(lse), _ptr(col_mass), _ptr(sink_idx),
                                   _ptr(workspace),
                                   0 if workspace is None else workspace.numel() * workspace.element_size(), _stream()))


def refresh_attn(q, k, v, shape: Shape, out, lse) -> None:
    """Dense attention of every row of q over every row of k / v (block-entry refresh)."""
    for t, name in ((q, "Q"), (k, "K"), (v, "V"), (out, "out")):
        _need(t, torch.bfloat16, name)
    _check(lib().focus_refresh_attn(_ptr(q), _ptr(k), _ptr(v), C.byref(shape), _ptr(out), _ptr(lse), _stream()))


def token_confidence_workspace(n_rows: int, vocab: int) -> int:
    return int(lib().focus_token_confidence_workspace(n_rows, vocab))


def token_confidence(logits, masked, tokens, conf, workspace) -> None:
    """logits bf16 [n_rows, vocab] (row stride a multiple of 8); workspace of token_confidence_workspace() bytes."""
    _need(logits, torch.bfloat16, "logits")
    _need(conf, torch.float32, "conf")
    if logits.stride(1) != 1:
        raise ValueError("logits: innermost stride must be 1")
    _check(lib().focus_token_confidence(_ptr(logits), logits.stride(0), _ptr(masked), logits.shape[0], logits.shape[1],
                                        _ptr(tokens), _ptr(conf), _ptr(workspace),
                                        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream()))


def cache_update(k_cache, v_cache, shape: Shape, k_new, v_new, active_idx, counts, row_base: int) -> None:
    """k_cache, v_cache bf16 [H, M+N, d] (strides from `shape`), k_new, v_new bf16 [H, max_active, d]."""
    for t, name in ((k_cache, "K_cache"), (v_cache, "V_cache"), (k_new, "K_new"), (v_new, "V_new")):
        _need(t, torch.bfloat16, name)
    if k_new.stride() != v_new.stride() or k_new.stride(2) != 1:
        raise ValueError("K_new and V_new must share their strides, innermost 1")
    _check(lib().focus_cache_update(_ptr(k_cache), _ptr(v_cache), C.byref(shape), _ptr(k_new), _ptr(v_new), k_new.stride(0),
                                    k_new.stride(1), _ptr(active_idx), _ptr(counts), active_idx.numel(), row_base, _stream()))


def cache_refresh(k_cache, v_cache, shape: Shape, k_new, v_new, kbar) -> None:
    """All rows of k_cache / v_cache bf16 [H, M+N, d] take k_new / v_new; kbar fp32 [H, n_b, d] (or None) gets the block means."""
    for t, name in ((k_cache, "K_cache"), (v_cache, "V_cache"), (k_new, "K_new"), (v_new, "V_new")):
        _need(t, torch.bfloat16, name)
    if kbar is not None:
        _need(kbar, torch.float32, "kbar")
    if k_new.stride() != v_new.stride() or k_new.stride(2) != 1:
        raise ValueError("K_new and V_new must share their strides, innermost 1")
    _check(lib().focus_cache_refresh(_ptr(k_cache), _ptr(v_cache), C.byref(shape), _ptr(k_new), _ptr(v_new), k_new.stride(0),
                                     k_new.stride(1), _ptr(kbar), _stream()))


def sparse_layer(q, focus_idx, active_idx, counts, k, v, kbar, shape: Shape, n_keep: int, sink_idx, n_sink: int, scores,
                 kept_blocks, out, lse, workspace) -> None:
    _need(q, torch.bfloat16, "Q")
    _need(k, torch.bfloat16, "K")
    _need(v, torch.bfloat16, "V")
    _need(out, torch.bfloat16, "out")
    _check(lib().focus_sparse_layer(_ptr(q), _ptr(focus_idx), _ptr(active_idx), _ptr(counts), focus_idx.numel(),
                                    active_idx.numel(), _ptr(k), _ptr(v), _ptr(kbar), C.byref(shape), n_keep, _ptr(sink_idx),
                                    n_sink, _ptr(scores), _ptr(kept_blocks), _ptr(out), _ptr(lse), _ptr(workspace),
                                    0 if workspace is None else workspace.numel() * workspace.element_size(), _stream()))


def sparse_layer_static(q, focus_idx, active_idx, counts, k, v, kbar, shape: Shape, n_keep: int, sink_idx, n_sink: int, scores,
                        kept_blocks, out, lse) -> None:
    """focus_sparse_layer without a workspace argument: the library's built-in scratch array is used; nothing is allocated."""
    _need(q, torch.bfloat16, "Q")
    _need(k, torch.bfloat16, "K")
    _need(v, torch.bfloat16, "V")
    _need(out, torch.bfloat16, "out")
    _check(lib().focus_sparse_layer_static(_ptr(q), _ptr(focus_idx), _ptr(active_idx), _ptr(counts), focus_idx.numel(),
                                           active_idx.numel(), _ptr(k), _ptr(v), _ptr(kbar), C.byref(shape), n_keep,
                                           _ptr(sink_idx), n_sink, _ptr(scores), _ptr(kept_blocks), _ptr(out), _ptr(lse),
                                           _stream()))
