"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every declared symbol, and
rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import pytest

from paper_2602_02159_amd import binding as fb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(fb.LIB_PATH):
        from paper_2602_02159_amd import build
        build.build(verbose=False)
    return fb.lib()


def _shape(**kw):
    s = fb.Shape()
    s.n_heads, s.head_dim, s.n_ctx, s.n_resp, s.block, s.n_gen = 4, 64, 1024, 32, 64, 32
    for n, rows in (("q", 32), ("k", 1056), ("v", 1056), ("o", 8)):
        setattr(s, n + "_stride_n", 64)
        setattr(s, n + "_stride_h", 64 * rows)
    for k, v in kw.items():
        setattr(s, k, v)
    return s


def test_every_declared_symbol_is_exported(L):
    header = open(os.path.join(ROOT, "include", "focus.h")).read()
    declared = set(re.findall(r"\b(focus_[a-z_]+)\s*\(", header))
    assert declared == set(fb.EXPORTS)
    for name in declared:
        assert hasattr(L, name), name
    assert L.focus_version().decode().startswith("focus-gfx950")


def test_host_helpers(L):
    assert fb.helper_k(4.0, 2) == 8 and fb.helper_k(0.5, 1) == 1 and fb.helper_k(0.25, 1) == 0 and fb.helper_k(1.5, 3) == 5
    assert [fb.helper_n_keep(a, n) for a, n in ((0.10, 64), (0.05, 128), (0.03, 256), (0.5, 7))] == [6, 6, 7, 3]
    assert fb.helper_n_sink(0.01, 32768) == 327 and fb.helper_n_sink(0.01, 8192) == 81


def test_workspace_sizes(L):
    s = _shape()
    assert fb.workspace_bytes(fb.FN_BLOCK_SCORES, s) >= 4 * 16 * 4 + 16 * 4     # per-head partials + scores
    assert fb.workspace_bytes(fb.FN_FIND_SINKS, s, 8) >= 4 * 1056 * 16 * 4
    assert fb.workspace_bytes(fb.FN_SPARSE_ATTN, s, 8, 4, 2) > 0
    assert fb.workspace_bytes(fb.FN_SPARSE_ATTN, s, 8, 17, 2) == 0      # n_keep > n_b
    assert fb.workspace_bytes(fb.FN_SPARSE_ATTN, s, 33, 4, 2) == 0      # more active rows than Q has
    assert fb.workspace_bytes(fb.FN_PROBE_LAYER, s, 8) >= 4 * 1056 * 16 * 4
    assert fb.workspace_bytes(99, s) == 0
    assert fb.workspace_bytes(fb.FN_FIND_SINKS, _shape(head_dim=96), 8) == 0


def test_bad_arguments_are_rejected_on_the_host(L):
    fake = C.c_void_p(4096)  # never dereferenced: validation fails first
    s = _shape()
    sp = C.byref(s)
    big = 1 << 40
    # select: NULL conf, k out of range, bad range, capacity too small for the window union
    assert L.focus_select_queries(None, None, 32, 8, 0, 0, 32, fake, fake, 8, fake, None) == fb.FOCUS_EINVAL
    assert L.focus_select_queries(fake, None, 32, 0, 0, 0, 32, fake, fake, 8, fake, None) == fb.FOCUS_EINVAL
    assert L.focus_select_queries(fake, None, 32, 33, 0, 0, 32, fake, fake, 33, fake, None) == fb.FOCUS_EINVAL
    assert L.focus_select_queries(fake, None, 32, 8, 0, 5, 5, fake, fake, 8, fake, None) == fb.FOCUS_EINVAL
    assert L.focus_select_queries(fake, None, 32, 8, 8, 0, 32, fake, fake, 31, fake, None) == fb.FOCUS_EINVAL
    assert L.focus_select_queries(fake, None, 20000, 8, 0, 0, 32, fake, fake, 8, fake, None) == fb.FOCUS_EINVAL
    assert "max_active" in fb.last_error() or "n_gen" in fb.last_error()
    # block means: unsupported head_dim, misaligned pointer, bad stride
    assert L.focus_block_means(fake, C.byref(_shape(head_dim=96)), fake, None) == fb.FOCUS_EUNSUPPORTED
    assert L.focus_block_means(C.c_void_p(4100), sp, fake, None) == fb.FOCUS_EINVAL
    assert L.focus_block_means(fake, C.byref(_shape(k_stride_n=60)), fake, None) == fb.FOCUS_EINVAL
    assert L.focus_block_means(fake, None, fake, None) == fb.FOCUS_EINVAL
    # block scores: n_keep out of range, no kbar and no K, missing workspace
    assert L.focus_block_scores(fake, fake, None, 8, fake, None, sp, 17, None, fake, fake, big, None) == fb.FOCUS_EINVAL
    assert L.focus_block_scores(fake, fake, None, 8, None, None, sp, 4, None, fake, fake, big, None) == fb.FOCUS_EINVAL
    assert L.focus_block_scores(fake, fake, None, 8, fake, None, sp, 4, None, fake, None, 0, None) == fb.FOCUS_EWORKSPACE
    assert L.focus_block_scores(fake, fake, None, 8, fake, None, sp, 4, None, fake, fake, 16, None) == fb.FOCUS_EWORKSPACE
    # the two halves of block scores: NULL output, neither kbar nor K, too many focus slots; bad part / keep counts
    assert L.focus_block_partials(fake, fake, None, 8, fake, None, sp, None, None) == fb.FOCUS_EINVAL
    assert L.focus_block_partials(fake, fake, None, 8, None, None, sp, fake, None) == fb.FOCUS_EINVAL
    assert L.focus_block_partials(fake, fake, None, 33, fake, None, sp, fake, None) == fb.FOCUS_EINVAL
    assert L.focus_top_blocks(fake, 0, None, 8, 16, 4, fake, fake, None) == fb.FOCUS_EINVAL
    assert L.focus_top_blocks(fake, 4, None, 8, 16, 17, fake, fake, None) == fb.FOCUS_EINVAL
    assert L.focus_top_blocks(fake, 4, None, 8, 16, 4, None, fake, None) == fb.FOCUS_EINVAL
    assert L.focus_top_blocks(fake, 4, None, 8, 16, 4, fake, None, None) == fb.FOCUS_EINVAL
    # confidence: NULL output, misaligned rows, bad stride; cache update: NULL pointer, bad stride of the new states
    assert L.focus_token_confidence(fake, 1000, None, 4, 1000, None, fake, fake, big, None) == fb.FOCUS_EINVAL
    assert L.focus_token_confidence(fake, 1001, None, 4, 1000, fake, fake, fake, big, None) == fb.FOCUS_EINVAL
    assert L.focus_token_confidence(fake, 992, None, 4, 1000, fake, fake, fake, big, None) == fb.FOCUS_EINVAL
    assert L.focus_token_confidence(fake, 1000, None, 0, 1000, fake, fake, fake, big, None) == fb.FOCUS_EINVAL
    assert L.focus_token_confidence(fake, 131072, None, 64, 131072, fake, fake, None, 0, None) == fb.FOCUS_EWORKSPACE
    assert fb.token_confidence_workspace(64, 131072) >= 64 * 16 * 12 and fb.token_confidence_workspace(0, 10) == 0
    assert L.focus_cache_update(fake, None, sp, fake, fake, 512, 64, fake, None, 8, 1024, None) == fb.FOCUS_EINVAL
    assert L.focus_cache_update(fake, fake, sp, fake, fake, 512, 60, fake, None, 8, 1024, None) == fb.FOCUS_EINVAL
    # refresh: NULL output, misaligned K
    assert L.focus_refresh_attn(fake, fake, fake, sp, None, None, None) == fb.FOCUS_EINVAL
    assert L.focus_refresh_attn(fake, C.c_void_p(4104), fake, sp, fake, None, None) == fb.FOCUS_EINVAL
    # group expansion: NULL list, non-positive group
    assert L.focus_expand_groups(None, 4, fake, 4, None, 32, 2, fake, fake, fake, None) == fb.FOCUS_EINVAL
    assert L.focus_expand_groups(fake, 4, fake, 4, None, 32, 0, fake, fake, fake, None) == fb.FOCUS_EINVAL
    # cache refresh: NULL source, source aliasing the cache, bad stride
    assert L.focus_cache_refresh(fake, fake, sp, None, fake, 4096, 128, None, None) == fb.FOCUS_EINVAL
    assert L.focus_cache_refresh(fake, fake, sp, fake, fake, 4096, 128, None, None) == fb.FOCUS_EINVAL
    assert L.focus_cache_refresh(fake, fake, sp, C.c_void_p(8192), C.c_void_p(12288), 4096, 100, None, None) == fb.FOCUS_EINVAL
    # probe layer: NULL V, n_sink out of range, workspace too small
    assert L.focus_probe_layer(fake, fake, None, 8, fake, None, sp, 2, fake, None, None, fake, fake, big, None) == fb.FOCUS_EINVAL
    assert L.focus_probe_layer(fake, fake, None, 8, fake, fake, sp, 5000, fake, None, None, fake, fake, big, None) == fb.FOCUS_EINVAL
    assert L.focus_probe_layer(fake, fake, None, 8, fake, fake, sp, 2, fake, None, None, fake, fake, 4096, None) == fb.FOCUS_EWORKSPACE
    # find sinks: n_sink out of range, workspace too small
    assert L.focus_find_sinks(fake, fake, None, 8, fake, sp, 2000, None, fake, fake, big, None) == fb.FOCUS_EINVAL
    assert L.focus_find_sinks(fake, fake, None, 8, fake, sp, 2, None, fake, fake, 1024, None) == fb.FOCUS_EWORKSPACE
    assert L.focus_find_sinks(fake, fake, None, 0, fake, sp, 2, None, fake, fake, big, None) == fb.FOCUS_EINVAL
    # sparse attention: NULL output, NULL index list with a non-zero count, zero shape
    assert L.focus_sparse_attn(fake, fake, None, 8, fake, fake, sp, fake, 4, fake, 2, None, None, fake, big, None) == fb.FOCUS_EINVAL
    assert L.focus_sparse_attn(fake, fake, None, 8, fake, fake, sp, None, 4, fake, 2, fake, None, fake, big, None) == fb.FOCUS_EINVAL
    assert L.focus_sparse_attn(fake, fake, None, 8, fake, fake, C.byref(_shape(n_heads=0)), fake, 4, fake, 2, fake, None,
                               fake, big, None) == fb.FOCUS_EINVAL
    assert L.focus_sparse_attn(fake, fake, None, 8, fake, fake, sp, fake, 4, fake, 2, fake, None, fake, 64, None) == fb.FOCUS_EWORKSPACE
    assert fb.last_error() != ""


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    """No silent fallback: without the built HIP library the binding raises, and so does everything on top of it."""
    monkeypatch.setattr(fb, "_lib", None)
    monkeypatch.setattr(fb, "LIB_PATH", str(tmp_path / "libfocus_hip.so"))
    with pytest.raises(FileNotFoundError):
        fb.lib()
    with pytest.raises(FileNotFoundError):
        fb.helper_k(4.0, 1)
