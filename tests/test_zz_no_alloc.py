"""focus_sparse_layer_static (the entry point for callers that cannot allocate) against focus_sparse_layer, through the C ABI."""
import ctypes as C

import numpy as np
import pytest
import torch

import focus_inputs as fi
from paper_2602_02159_amd import binding as fb

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _layer(seed, H, M, N, d, n_gen):
    g = torch.Generator().manual_seed(seed)
    mk = lambda r: torch.randn(H, r, d, generator=g).to(torch.bfloat16).to(DEV)
    return mk(n_gen), mk(M + N), mk(M + N)


def _both(q, k, v, M, B, focus, active, counts, n_keep, sinks, kbar):
    """One call of each entry point on the same inputs, straight through ctypes; returns the two sets of outputs."""
    L = fb.lib()
    H, n_gen, d = q.shape
    n_b = -(-M // B)
    n_sink = sinks.numel()
    res = []
    for static in (False, True):
        out = torch.full((H, active.numel(), d), float("nan"), dtype=torch.bfloat16, device=DEV)
        lse = torch.full((H, active.numel()), float("nan"), dtype=torch.float32, device=DEV)
        scores = torch.full((n_b,), float("nan"), dtype=torch.float32, device=DEV)
        kept = torch.full((max(n_keep, 1),), -7, dtype=torch.int32, device=DEV)
        s = fb.make_shape(q, k, v, M, B, out)
        p = lambda t: None if t is None else C.c_void_p(t.data_ptr())
        common = (p(q), p(focus), p(active), p(counts), focus.numel(), active.numel(), p(k), p(v), p(kbar), C.byref(s), n_keep,
                  p(sinks), n_sink, p(scores), p(kept), p(out), p(lse))
        stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
        if static:
            rc = L.focus_sparse_layer_static(*common, stream)
        else:
            nbytes = fb.workspace_bytes(fb.FN_SPARSE_LAYER, s, active.numel(), n_keep, n_sink)
            ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=DEV).fill_(0x5A)
            rc = L.focus_sparse_layer(*common, p(ws), ws.numel(), stream)
        assert rc == 0, fb.last_error()
        torch.cuda.synchronize()
        res.append((scores, kept, out, lse))
    return res


def _same(a, b, n_q):
    (s0, k0, o0, l0), (s1, k1, o1, l1) = a, b
    assert torch.equal(s0, s1) and torch.equal(k0, k1)                     # scores and kept blocks: bit-exact
    assert torch.equal(o0[:, :n_q], o1[:, :n_q]) and torch.equal(l0[:, :n_q], l1[:, :n_q])   # same kernels, same split plan
    assert not torch.isnan(o1[:, :n_q].float()).any()


def test_static_scratch_entry_point_matches_the_workspace_one_twice_in_a_row():
    assert torch.cuda.is_available()
    # first call: the 32K-context layer of the benchmark (16 queries, 7 of 256 blocks, 4 sinks), block means cached
    w = fi.CTX32K
    q, k, v = fi.layer_qkv(w, 0, DEV)
    n_b = w.n_blocks
    kbar = torch.empty(w.n_heads, n_b, w.head_dim, dtype=torch.float32, device=DEV)
    fb.block_means(k, fb.make_shape(q, k, None, w.n_ctx, w.block), kbar)
    rng = np.random.default_rng(5)
    focus = torch.tensor(np.sort(rng.choice(w.n_gen, 16, replace=False)).astype(np.int32), device=DEV)
    counts = torch.tensor([16, 16], dtype=torch.int32, device=DEV)
    sinks = torch.tensor([0, 1, 8191, 20000], dtype=torch.int32, device=DEV)
    a, b = _both(q, k, v, w.n_ctx, w.block, focus, focus, counts, w.n_keep, sinks, kbar)
    _same(a, b, 16)
    # second call, smaller: fewer heads, a ragged context, fewer queries than slots, scores from raw K (kbar = NULL);
    # the array still holds the first call's partial results
    H, M, N, d, B, n_gen = 3, 1000, 37, 64, 48, 40
    q2, k2, v2 = _layer(9, H, M, N, d, n_gen)
    focus2 = torch.tensor([2, 5, 11, 30, -1, -1], dtype=torch.int32, device=DEV)
    active2 = torch.tensor([1, 2, 3, 5, 11, 12, 30, 31, -1, -1, -1, -1], dtype=torch.int32, device=DEV)
    counts2 = torch.tensor([4, 8], dtype=torch.int32, device=DEV)
    sinks2 = torch.tensor([7, 500, 999], dtype=torch.int32, device=DEV)
    a2, b2 = _both(q2, k2, v2, M, B, focus2, active2, counts2, 5, sinks2, None)
    _same(a2, b2, 8)
    # and the first shape once more: nothing of the smaller call is left behind that matters
    a3, b3 = _both(q, k, v, w.n_ctx, w.block, focus, focus, counts, w.n_keep, sinks, kbar)
    _same(a3, b3, 16)
    assert torch.equal(a[2], b3[2])


def test_static_scratch_entry_point_rejects_shapes_beyond_its_array():
    # 64 active queries over half of 512 blocks (the paper's own hyper-parameters at 32K) need more than 8 MiB of partial results
    L = fb.lib()
    H, M, N, d, B, n_gen = 32, 32768, 64, 128, 64, 64
    q = torch.zeros(H, n_gen, d, dtype=torch.bfloat16, device=DEV)
    k = torch.zeros(H, M + N, d, dtype=torch.bfloat16, device=DEV)
    out = torch.full((H, n_gen, d), 3.0, dtype=torch.bfloat16, device=DEV)
    s = fb.make_shape(q, k, k, M, B, out)
    assert fb.workspace_bytes(fb.FN_SPARSE_LAYER, s, n_gen, 256, 327) > (8 << 20)
    idx = torch.arange(n_gen, dtype=torch.int32, device=DEV)
    kept = torch.full((256,), -7, dtype=torch.int32, device=DEV)
    sinks = torch.arange(327, dtype=torch.int32, device=DEV)
    p = lambda t: C.c_void_p(t.data_ptr())
    rc = L.focus_sparse_layer_static(p(q), p(idx), p(idx), None, n_gen, n_gen, p(k), p(k), None, C.byref(s), 256, p(sinks), 327,
                                     None, p(kept), p(out), None, None)
    assert rc == fb.FOCUS_EWORKSPACE and "8388608" in fb.last_error()
    torch.cuda.synchronize()
    assert (out == 3.0).all() and (kept == -7).all()                       # nothing was enqueued
