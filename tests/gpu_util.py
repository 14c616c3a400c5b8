"""Helpers for the GPU parity tests: buffer allocation around the C-ABI calls and oracle-side conversions.
Only marshalling lives here; every step of the method runs inside the library."""
from __future__ import annotations

import numpy as np
import torch

from oracle import focus_oracle as fo
from paper_2602_02159_amd import binding as fb

DEV = "cuda:0"
CANARY = -7777


def to_np(t: torch.Tensor) -> np.ndarray:
    """bf16/fp32 tensor -> float32 numpy (exact widening for bf16)."""
    return t.detach().float().cpu().numpy()


def i32(x, n=None, fill=CANARY):
    """int32 device buffer holding x (list/array) or a canary-filled buffer of n entries."""
    if x is None:
        return torch.full((n,), fill, dtype=torch.int32, device=DEV)
    return torch.tensor(np.asarray(x, dtype=np.int32), dtype=torch.int32, device=DEV)


def ws(nbytes: int) -> torch.Tensor:
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=DEV)


def gpu_select(conf, masked, k, window, lo, hi, max_active=None):
    conf_d = torch.as_tensor(conf, dtype=torch.float32).to(DEV)
    masked_d = None if masked is None else torch.as_tensor(masked, dtype=torch.uint8).to(DEV)
    if max_active is None:
        max_active = min(hi - lo, k * (2 * (window // 2) + 1))
    focus = i32(None, k)
    active = i32(None, max_active)
    counts = i32(None, 2)
    fb.select_queries(conf_d, masked_d, k, window, lo, hi, focus, active, counts)
    torch.cuda.synchronize()
    return focus, active, counts


def gpu_block_means(k, n_ctx, block):
    H, L, d = k.shape
    s = fb.make_shape(k[:, :1], k, None, n_ctx, block)
    n_b = -(-n_ctx // block)
    kbar = torch.full((H, n_b, d), float("nan"), dtype=torch.float32, device=DEV)
    fb.block_means(k, s, kbar)
    torch.cuda.synchronize()
    return kbar


def gpu_block_scores(q, focus, counts, k, kbar, n_ctx, block, n_keep):
    s = fb.make_shape(q, k, None, n_ctx, block)
    n_b = -(-n_ctx // block)
    scores = torch.full((n_b,), float("nan"), dtype=torch.float32, device=DEV)
    kept = i32(None, max(n_keep, 1))
    w = ws(fb.workspace_bytes(fb.FN_BLOCK_SCORES, s))
    fb.block_scores(q, focus, counts, k, kbar, s, n_keep, scores, kept, w)
    torch.cuda.synchronize()
    return scores, kept[:n_keep]


def gpu_find_sinks(q, active, counts, k, n_ctx, block, n_sink):
    s = fb.make_shape(q, k, None, n_ctx, block)
    L = k.shape[1]
    col = torch.full((L,), float("nan"), dtype=torch.float32, device=DEV)
    sinks = i32(None, max(n_sink, 1))
    w = ws(fb.workspace_bytes(fb.FN_FIND_SINKS, s, active.numel()))
    fb.find_sinks(q, active, counts, k, s, n_sink, col, sinks, w)
    torch.cuda.synchronize()
    return col, sinks[:n_sink]


def gpu_sparse_attn(q, active, counts, k, v, n_ctx, block, kept, sinks, want_lse=True, out=None):
    H, _, d = q.shape
    n_keep = 0 if kept is None else kept.numel()
    n_sink = 0 if sinks is None else sinks.numel()
    max_active = active.numel()
    if out is None:
        out = torch.full((H, max_active, d), float("nan"), dtype=torch.bfloat16, device=DEV)
    lse = torch.full((H, max_active), float("nan"), dtype=torch.float32, device=DEV) if want_lse else None
    s = fb.make_shape(q, k, v, n_ctx, block, out)
    w = ws(fb.workspace_bytes(fb.FN_SPARSE_ATTN, s, max_active, n_keep, n_sink))
    fb.sparse_attn(q, active, counts, k, v, s, kept if n_keep else None, n_keep, sinks if n_sink else None, n_sink, out,
                   lse, w)
    torch.cuda.synchronize()
    return out, lse


def assert_attention_close(out_gpu: torch.Tensor, out_ref: np.ndarray, max_abs=2e-2, mean_abs=2e-3):
    """The stated bar for bf16 attention outputs against the fp64 oracle."""
    diff = np.abs(to_np(out_gpu).astype(np.float64) - out_ref)
    assert np.isfinite(diff).all()
    assert diff.max() <= max_abs, f"max abs err {diff.max():.3e}"
    assert diff.mean() <= mean_abs, f"mean abs err {diff.mean():.3e}"


def oracle_layer(q, k, v, focus, active, sinks, n_ctx, block, n_keep):
    return fo.focus_layer(to_np(q), to_np(k), to_np(v), focus, active, sinks, n_ctx, block, n_keep)


def gpu_sparse_layer(q, focus, active, counts, k, v, kbar, n_ctx, block, n_keep, sinks):
    H, _, d = q.shape
    n_sink = 0 if sinks is None else sinks.numel()
    n_b = -(-n_ctx // block)
    max_active = active.numel()
    out = torch.full((H, max_active, d), float("nan"), dtype=torch.bfloat16, device=DEV)
    lse = torch.full((H, max_active), float("nan"), dtype=torch.float32, device=DEV)
    scores = torch.full((n_b,), float("nan"), dtype=torch.float32, device=DEV)
    kept = i32(None, max(n_keep, 1))
    s = fb.make_shape(q, k, v, n_ctx, block, out)
    w = ws(fb.workspace_bytes(fb.FN_SPARSE_LAYER, s, max_active, n_keep, n_sink))
    w.fill_(0xAB)   # the call must not rely on a cleared workspace
    fb.sparse_layer(q, focus, active, counts, k, v, kbar, s, n_keep, sinks if n_sink else None, n_sink, scores, kept, out, lse, w)
    torch.cuda.synchronize()
    return scores, kept[:n_keep], out, lse


def gpu_probe_layer(q, active, counts, k, v, n_ctx, block, n_sink):
    H, _, d = q.shape
    L = k.shape[1]
    max_active = active.numel()
    out = torch.full((H, max_active, d), float("nan"), dtype=torch.bfloat16, device=DEV)
    lse = torch.full((H, max_active), float("nan"), dtype=torch.float32, device=DEV)
    col = torch.full((L,), float("nan"), dtype=torch.float32, device=DEV)
    sinks = i32(None, max(n_sink, 1))
    s = fb.make_shape(q, k, v, n_ctx, block, out)
    w = ws(fb.workspace_bytes(fb.FN_PROBE_LAYER, s, max_active))
    w.fill_(0xCD)
    fb.probe_layer(q, active, counts, k, v, s, n_sink, out, lse, col, sinks, w)
    torch.cuda.synchronize()
    return out, lse, col, sinks[:n_sink]
