"""The oracle's pins must be able to fail: each case plants one plausible mistake in the oracle (on the CPU,
by patching one of its functions) and checks that at least one pin of tests/test_oracle_pins.py rejects it."""
import math

import numpy as np
import pytest

from oracle import focus_oracle as fo
from tests import test_oracle_pins as pins

_f64 = lambda x: np.asarray(x, dtype=np.float64)


def _pins_reject(monkeypatch, name, broken, checks):
    monkeypatch.setattr(fo, name, broken)
    for check in checks:
        try:
            check()
        except AssertionError:
            return True
    return False


def test_missing_softmax_scale_is_caught(monkeypatch):
    def broken(Q, active, K, V, index_set, n_ctx):
        d = K.shape[2]
        return orig(Q * math.sqrt(d) ** 0.5, active, K * math.sqrt(d) ** 0.5, V, index_set, n_ctx)   # logits without 1/sqrt(d)
    orig = fo.sparse_attention
    assert _pins_reject(monkeypatch, "sparse_attention", broken,
                        [pins.test_dense_reduction_equals_full_bidirectional_attention])


def test_dropping_the_response_rows_is_caught(monkeypatch):
    orig = fo.sparse_attention

    def broken(Q, active, K, V, index_set, n_ctx):
        return orig(Q, active, K[:, :n_ctx], V[:, :n_ctx], index_set, n_ctx)
    assert _pins_reject(monkeypatch, "sparse_attention", broken,
                        [pins.test_dense_reduction_equals_full_bidirectional_attention])


def test_union_without_dedupe_is_caught(monkeypatch):
    def broken(sinks, blocks, n_ctx, block):
        rows = [int(j) for j in sinks if 0 <= j < n_ctx]
        for b in blocks:
            if 0 <= b < -(-n_ctx // block):
                rows += list(range(b * block, min((b + 1) * block, n_ctx)))
        return np.array(sorted(rows), dtype=np.int64)
    assert _pins_reject(monkeypatch, "attention_index_set", broken,
                        [pins.test_attention_index_set_membership, pins.test_sparse_attention_metamorphic])


def test_tie_to_the_higher_index_is_caught(monkeypatch):
    def broken(values, n, candidates=None):
        v = _f64(values).ravel() + 0.0
        idx = np.arange(v.size)
        if candidates is not None:
            idx = idx[np.asarray(candidates, dtype=bool).ravel()]
        vv = v[idx]
        nan = np.isnan(vv)
        order = np.lexsort((-idx, np.where(nan, 0.0, -vv), nan))
        return np.sort(idx[order[: max(0, min(n, idx.size))]]).astype(np.int64)
    assert _pins_reject(monkeypatch, "top_indices", broken,
                        [pins.test_top_indices_exhaustive_small, pins.test_top_indices_special_values])


def test_block_mean_over_nominal_block_size_is_caught(monkeypatch):
    def broken(K, n_ctx, block):
        H, _, d = K.shape
        n_b = -(-n_ctx // block)
        out = np.empty((H, n_b, d))
        for h in range(H):
            for b in range(n_b):
                out[h, b] = _f64(K[h, b * block:min((b + 1) * block, n_ctx)]).sum(axis=0) / block
        return out
    assert _pins_reject(monkeypatch, "block_means", broken, [pins.test_block_means_brute_force_ragged_tail])


def test_block_mean_including_response_rows_is_caught(monkeypatch):
    def broken(K, n_ctx, block):
        H, L, d = K.shape
        n_b = -(-n_ctx // block)
        out = np.empty((H, n_b, d))
        for h in range(H):
            for b in range(n_b):
                out[h, b] = _f64(K[h, b * block:(b + 1) * block]).mean(axis=0)     # runs past M into the response
        return out
    assert _pins_reject(monkeypatch, "block_means", broken, [pins.test_block_means_brute_force_ragged_tail])


@pytest.mark.parametrize("variant", ["sum_over_focus", "scaled"])
def test_wrong_relevance_aggregation_is_caught(monkeypatch, variant):
    def broken(Q, focus, kbar):
        focus = np.asarray(focus, dtype=np.int64)
        R = np.zeros(kbar.shape[1])
        for h in range(Q.shape[0]):
            q = _f64(Q[h])[focus]
            q_bar = q.sum(axis=0) if variant == "sum_over_focus" else q.mean(axis=0) / math.sqrt(Q.shape[2])
            R += kbar[h] @ q_bar
        return R / Q.shape[0]
    assert _pins_reject(monkeypatch, "block_relevance", broken,
                        [pins.test_block_relevance_scale_closed_form, pins.test_block_relevance_is_mean_of_pairwise_dot_products])


@pytest.mark.parametrize("variant", ["prompt_only_softmax", "sum_over_heads", "no_scale"])
def test_wrong_sink_score_is_caught(monkeypatch, variant):
    def broken(Q, active, K, pooled_query=False):
        active = np.asarray(active, dtype=np.int64)
        H, L, d = K.shape
        S = np.zeros(L)
        for h in range(H):
            q = _f64(Q[h])[active]
            logits = q @ _f64(K[h]).T / (1.0 if variant == "no_scale" else math.sqrt(d))
            if variant == "prompt_only_softmax":
                logits[:, L - 2:] = -np.inf           # pretend the last rows are not part of the softmax
            p = np.exp(logits - logits.max(axis=1, keepdims=True))
            p /= p.sum(axis=1, keepdims=True)
            S += p.mean(axis=0)
        return S if variant == "sum_over_heads" else S / H
    assert _pins_reject(monkeypatch, "sink_scores", broken,
                        [pins.test_sink_scores_brute_force_definition, pins.test_sink_scores_against_torch_softmax_and_row_sums])


def test_window_of_full_width_is_caught(monkeypatch):
    def broken(focus, w, lo, hi):
        s = set()
        for i in np.asarray(focus).tolist():
            for l in range(i - w, i + w + 1):       # +-w instead of +-floor(w/2)
                if lo <= l < hi:
                    s.add(l)
        return np.array(sorted(s), dtype=np.int64)
    assert _pins_reject(monkeypatch, "expand_window", broken,
                        [pins.test_expand_window_paper_default_is_nine_wide, lambda: pins.test_expand_window_brute_force(0)])


def test_sinks_among_response_rows_are_caught(monkeypatch):
    assert _pins_reject(monkeypatch, "select_sinks", lambda S, n_ctx, n_sink: fo.top_indices(S, n_sink),
                        [pins.test_select_sinks_only_prompt_positions])


def test_recomputing_sinks_per_layer_is_caught(monkeypatch):
    orig = fo.focus_step

    def broken(*a, **kw):
        r = orig(*a, **kw)
        for lay in r["layers"].values():
            lay["sinks_used"] = r["sinks"].copy()     # equal values, but not the array handed down
        return r
    assert _pins_reject(monkeypatch, "focus_step", broken, [pins.test_step_reuses_probe_layer_sinks_unchanged])


@pytest.mark.parametrize("variant", ["max_logit", "tie_high", "ignore_mask"])
def test_wrong_token_confidence_is_caught(monkeypatch, variant):
    def broken(logits, masked=None):
        x = _f64(logits)
        tok, conf = np.full(len(x), -1, dtype=np.int64), np.zeros(len(x))
        for i, row in enumerate(x):
            if variant != "ignore_mask" and masked is not None and not masked[i]:
                continue
            m = row.max()
            hits = np.flatnonzero(row == m)
            tok[i] = int(hits[-1] if variant == "tie_high" else hits[0])
            conf[i] = m if variant == "max_logit" else 1.0 / np.exp(row - m).sum()     # the logit instead of the probability
        return tok, conf
    assert _pins_reject(monkeypatch, "token_confidence", broken,
                        [pins.test_token_confidence_closed_forms, pins.test_token_confidence_invariances_and_mask])


def test_cache_update_at_the_wrong_rows_is_caught(monkeypatch):
    def broken(K_cache, V_cache, K_new, V_new, active, row_base):
        K_out, V_out = np.array(K_cache, copy=True), np.array(V_cache, copy=True)
        for a, i in enumerate(active):
            K_out[:, i, :] = K_new[:, a, :]        # block-relative position used as a cache row
            V_out[:, i, :] = V_new[:, a, :]
        return K_out, V_out
    assert _pins_reject(monkeypatch, "cache_update", broken, [pins.test_cache_update_touches_exactly_the_refreshed_rows])
