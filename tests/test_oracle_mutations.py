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


def _decode_block_with_a_mistake(mistake):
    """decode_block re-stated with one planted mistake: 'update_after' (the new states reach the cache only after the
    layer has attended), 'no_persist' (every step starts again from the block-entry cache), 'sparse_skip' (sparse layers
    never write their new states), 'entry_prompt_only' (the block entry rewrites the prompt rows only)."""
    def broken(entry, steps, n_layers, l_dense, dense_tail, n_ctx, row_base, block, window, lo, hi, n_keep, n_sink):
        K0, V0, entry_out = [], [], []
        for l in range(n_layers):
            Q_all, K_all, V_all = entry(l)
            K, V = np.array(K_all, dtype=np.float64), np.array(V_all, dtype=np.float64)
            if mistake == "entry_prompt_only":
                K[:, n_ctx:], V[:, n_ctx:] = 0.0, 0.0
            K0.append(K)
            V0.append(V)
            entry_out.append(fo.full_attention(Q_all, np.arange(K.shape[1]), K, V)[0])
        Kc, Vc = [k.copy() for k in K0], [v.copy() for v in V0]
        out_steps = []
        for st in steps:
            if mistake == "no_persist":
                Kc, Vc = [k.copy() for k in K0], [v.copy() for v in V0]
            focus = fo.select_focus(st["conf"], st.get("masked"), st["k"])
            active = fo.expand_window(focus, window, lo, hi)
            sinks, S, per_layer = None, None, []
            for l in range(n_layers):
                Q, K_new, V_new = st["layer"](l)
                dense = l <= l_dense or l >= n_layers - dense_tail
                upd = lambda: fo.cache_update(Kc[l], Vc[l], _f64(K_new), _f64(V_new), active, row_base)
                if mistake != "update_after" and not (mistake == "sparse_skip" and not dense):
                    Kc[l], Vc[l] = upd()
                if dense:
                    o, lse = fo.full_attention(Q, active, Kc[l], Vc[l])
                    rec = {"kind": "dense", "out": o, "lse": lse}
                    if l == l_dense:
                        S = fo.sink_scores(Q, active, Kc[l])
                        sinks = fo.select_sinks(S, n_ctx, n_sink)
                else:
                    rec = fo.focus_layer(Q, Kc[l], Vc[l], focus, active, sinks, n_ctx, block, n_keep)
                    rec["kind"] = "sparse"
                if mistake == "update_after":
                    Kc[l], Vc[l] = upd()
                per_layer.append(rec)
            out_steps.append({"focus": focus, "active": active, "S": S, "sinks": sinks, "layers": per_layer})
        return {"entry": entry_out, "steps": out_steps, "K_cache": Kc, "V_cache": Vc}
    return broken


def test_the_restated_block_driver_without_a_mistake_passes_the_pins(monkeypatch):
    # the harness itself: with no mistake planted the restatement must be accepted, or the cases below prove nothing
    assert not _pins_reject(monkeypatch, "decode_block", _decode_block_with_a_mistake(None),
                            [pins.test_decode_block_entry_is_dense_bidirectional_attention_of_every_position,
                             pins.test_decode_block_step_equals_a_from_scratch_step_on_the_updated_cache,
                             pins.test_decode_block_cache_rows_persist_and_prompt_means_stay_frozen,
                             pins.test_decode_block_refreshed_positions_are_attended_with_their_new_states])


@pytest.mark.parametrize("mistake,pin", [
    ("update_after", "test_decode_block_refreshed_positions_are_attended_with_their_new_states"),
    ("no_persist", "test_decode_block_cache_rows_persist_and_prompt_means_stay_frozen"),
    ("sparse_skip", "test_decode_block_cache_rows_persist_and_prompt_means_stay_frozen"),
    ("entry_prompt_only", "test_decode_block_entry_is_dense_bidirectional_attention_of_every_position"),
])
def test_mistakes_in_the_block_driver_are_caught(monkeypatch, mistake, pin):
    assert _pins_reject(monkeypatch, "decode_block", _decode_block_with_a_mistake(mistake), [getattr(pins, pin)])
