"""Pins for the CPU oracle: each check ties an oracle function to something other than itself —
an independent library routine on a special case, a brute-force evaluation of the paper's
definition on tiny inputs, a closed form, or an invariance the mathematics fixes.
All CPU-only."""
import itertools
import math

import numpy as np
import pytest
import torch

from oracle import focus_oracle as fo


def _rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


# --------------------------------------------------------------------------- top-k total order (Eq. 4, Top-C, Top-N_sink)
def _brute_top(values, n, cand=None):
    items = [(i, float(v) + 0.0) for i, v in enumerate(values) if cand is None or cand[i]]
    items.sort(key=lambda t: (math.isnan(t[1]), -t[1] if not math.isnan(t[1]) else 0.0, t[0]))
    return sorted(i for i, _ in items[:n])


@pytest.mark.parametrize("seed", range(6))
def test_top_indices_matches_brute_force_sort(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 40))
    v = rng.integers(0, 6, n).astype(np.float64)  # many ties
    cand = rng.random(n) < 0.7
    for k in (0, 1, n // 2, n, n + 3):
        assert fo.top_indices(v, k).tolist() == _brute_top(v, k)
        assert fo.top_indices(v, k, cand).tolist() == _brute_top(v, k, cand)


def test_top_indices_exhaustive_small():
    # every length-4 vector over {0,1,2}: the kept set is exactly the k first of the stable descending sort
    for vals in itertools.product([0.0, 1.0, 2.0], repeat=4):
        for k in range(5):
            assert fo.top_indices(vals, k).tolist() == _brute_top(vals, k)


def test_top_indices_special_values():
    v = np.array([np.nan, -np.inf, -0.0, 0.0, np.inf, 1.0, np.nan])
    assert fo.top_indices(v, 1).tolist() == [4]
    assert fo.top_indices(v, 3).tolist() == [2, 4, 5]        # -0.0 ties +0.0: lower index wins
    assert fo.top_indices(v, 5).tolist() == [1, 2, 3, 4, 5]  # -inf still beats NaN
    assert fo.top_indices(v, 6).tolist() == [0, 1, 2, 3, 4, 5]
    assert fo.top_indices(np.zeros(5), 2).tolist() == [0, 1]  # all equal: lowest indices


def test_top_indices_agrees_with_torch_topk_when_no_ties():
    v = _rand(3, 257)
    got = fo.top_indices(v, 17)
    ref = torch.topk(torch.from_numpy(v), 17).indices.sort().values.numpy()
    assert got.tolist() == ref.tolist()


def test_nested_top_sets():
    v = _rand(4, 100)
    prev = set()
    for k in range(0, 101, 7):
        cur = set(fo.top_indices(v, k).tolist())
        assert prev <= cur and len(cur) == k
        prev = cur


def test_decision_margin():
    v = np.array([5.0, 1.0, 4.0, 0.0])
    assert fo.decision_margin(v, 2) == pytest.approx((4.0 - 1.0) / 5.0)
    assert fo.decision_margin(v, 4) == math.inf
    assert fo.decision_margin(np.array([1.0, 1.0, 0.0]), 1) == 0.0


# --------------------------------------------------------------------------- stage 1 (Eq. 4, Eq. 5)
def test_select_focus_masked_subset_and_clipping():
    conf = np.array([0.9, 0.1, 0.8, 0.8, 0.3, 0.95], dtype=np.float32)
    masked = np.array([1, 1, 1, 1, 1, 0], dtype=np.uint8)      # position 5 is already unmasked
    assert fo.select_focus(conf, masked, 2).tolist() == [0, 2]  # 0.8 tie -> lower position
    assert fo.select_focus(conf, masked, 3).tolist() == [0, 2, 3]
    assert fo.select_focus(conf, masked, 9).tolist() == [0, 1, 2, 3, 4]  # k clipped to #masked
    assert fo.select_focus(conf, None, 1).tolist() == [5]


@pytest.mark.parametrize("seed", range(5))
def test_expand_window_brute_force(seed):
    rng = np.random.default_rng(100 + seed)
    n = 40
    focus = np.sort(rng.choice(n, size=6, replace=False))
    for w in (0, 1, 2, 3, 8, 9):
        lo, hi = 3, 35
        got = fo.expand_window(focus, w, lo, hi)
        ref = [l for l in range(lo, hi) if any(abs(l - int(i)) <= w // 2 for i in focus)]
        assert got.tolist() == ref
        assert len(got) <= min(hi - lo, len(focus) * (2 * (w // 2) + 1))
    inside = focus[(focus >= 3) & (focus < 35)]
    assert fo.expand_window(focus, 0, 3, 35).tolist() == inside.tolist()
    assert fo.expand_window(focus, 1, 3, 35).tolist() == inside.tolist()


def test_expand_window_paper_default_is_nine_wide():
    assert fo.expand_window([20], 8, 0, 64).tolist() == list(range(16, 25))


# --------------------------------------------------------------------------- stage 2a (block means, Eq. 7)
def test_block_means_brute_force_ragged_tail():
    H, M, N, d, B = 2, 23, 5, 3, 8   # blocks of 8, 8, 7 prompt rows; 5 response rows must be ignored
    K = _rand(7, H, M + N, d)
    kb = fo.block_means(K, M, B)
    assert kb.shape == (H, 3, d)
    for h in range(H):
        for b in range(3):
            rows = range(b * B, min((b + 1) * B, M))
            for c in range(d):
                ref = sum(K[h, j, c] for j in rows) / len(rows)
                assert kb[h, b, c] == pytest.approx(ref, abs=1e-14)


def test_block_relevance_is_mean_of_pairwise_dot_products():
    # linearity: q_bar . K_bar_b equals the mean over (i in focus, j in block) of Q_i . K_j, averaged over heads
    H, M, N, d, B, n_gen = 3, 20, 4, 5, 6, 7
    Q, K = _rand(8, H, n_gen, d), _rand(9, H, M + N, d)
    focus = np.array([1, 4, 5])
    R = fo.block_relevance(Q, focus, fo.block_means(K, M, B))
    for b in range(4):
        rows = list(range(b * B, min((b + 1) * B, M)))
        acc = 0.0
        for h in range(H):
            for i in focus:
                for j in rows:
                    acc += sum(Q[h, i, c] * K[h, j, c] for c in range(d))
        assert R[b] == pytest.approx(acc / (H * len(focus) * len(rows)), abs=1e-13)


def test_block_relevance_scale_closed_form():
    # all queries e_0, block b's keys all (b+1)*e_0  =>  R_b = b+1 exactly: no hidden 1/sqrt(d) or 1/|focus|
    H, d, B, n_b = 4, 8, 5, 3
    Q = np.zeros((H, 6, d)); Q[..., 0] = 1.0
    K = np.zeros((H, n_b * B + 2, d))
    for b in range(n_b):
        K[:, b * B:(b + 1) * B, 0] = b + 1
    R = fo.block_relevance(Q, [0, 2, 3], fo.block_means(K, n_b * B, B))
    assert R.tolist() == [1.0, 2.0, 3.0]
    assert fo.select_blocks(R, 2).tolist() == [1, 2]


# --------------------------------------------------------------------------- stage 2b (Eq. 6)
def test_sink_scores_brute_force_definition():
    H, L, d, n_gen = 2, 6, 3, 4
    Q, K = _rand(10, H, n_gen, d), _rand(11, H, L, d)
    active = [0, 3]
    S = fo.sink_scores(Q, active, K)
    ref = [0.0] * L
    for h in range(H):
        for i in active:
            logit = [sum(Q[h, i, c] * K[h, j, c] for c in range(d)) / math.sqrt(d) for j in range(L)]
            z = sum(math.exp(x) for x in logit)
            for j in range(L):
                ref[j] += math.exp(logit[j]) / z / (H * len(active))
    assert np.allclose(S, ref, atol=1e-14)


def test_sink_scores_against_torch_softmax_and_row_sums():
    H, L, d, n_gen = 3, 50, 16, 9
    Q, K = _rand(12, H, n_gen, d), _rand(13, H, L, d)
    active = np.array([0, 2, 7, 8])
    S = fo.sink_scores(Q, active, K)
    tq, tk = torch.from_numpy(Q)[:, active], torch.from_numpy(K)
    P = torch.softmax(tq @ tk.transpose(1, 2) / math.sqrt(d), dim=-1)
    assert np.allclose(S, P.mean(dim=(0, 1)).numpy(), atol=1e-14)
    assert S.sum() == pytest.approx(1.0, abs=1e-12)           # every softmax row sums to one
    assert (S > 0).all()


def test_sink_scores_closed_forms():
    H, L, d = 2, 12, 4
    Q = _rand(14, H, 5, d)
    K = np.tile(_rand(15, 1, 1, d), (H, L, 1))               # all keys equal -> uniform attention
    S = fo.sink_scores(Q, [1, 2], K)
    assert np.allclose(S, 1.0 / L, atol=1e-15)
    assert fo.select_sinks(S + 0.0, 10, 3).tolist() == [0, 1, 2]
    # one key aligned with every query with a huge logit -> all mass on it
    Q2 = np.zeros((H, 3, d)); Q2[..., 0] = 30.0
    K2 = np.zeros((H, L, d)); K2[:, 7, 0] = 30.0
    S2 = fo.sink_scores(Q2, [0, 1, 2], K2)
    assert S2[7] == pytest.approx(1.0, abs=1e-12)
    assert fo.select_sinks(S2, L - 2, 1).tolist() == [7]


def test_select_sinks_only_prompt_positions():
    S = np.array([0.1, 0.3, 0.05, 0.2, 0.9, 0.8])  # last two are response rows
    assert fo.select_sinks(S, 4, 2).tolist() == [1, 3]


def test_sink_scores_key_shift_and_head_permutation_invariance():
    H, L, d = 3, 20, 8
    Q, K = _rand(16, H, 6, d), _rand(17, H, L, d)
    S = fo.sink_scores(Q, [0, 5], K)
    # adding one vector to every key shifts each row's logits by a constant: the softmax does not move
    assert np.allclose(fo.sink_scores(Q, [0, 5], K + _rand(18, 1, 1, d)), S, atol=1e-13)
    perm = [2, 0, 1]
    assert np.allclose(fo.sink_scores(Q[perm], [0, 5], K[perm]), S, atol=1e-15)
    # the other reading (pool the queries first) is a different quantity
    assert not np.allclose(fo.sink_scores(Q, [0, 5], K, pooled_query=True), S, atol=1e-6)


def test_sink_scores_pooled_query_reading_by_loops():
    # the other reading of Eq. 6 (kept for comparison only): per head ONE softmax of the mean active query
    H, L, d = 2, 9, 4
    Q, K = _rand(61, H, 5, d), _rand(62, H, L, d)
    active = [1, 3, 4]
    S = fo.sink_scores(Q, active, K, pooled_query=True)
    ref = np.zeros(L)
    for h in range(H):
        qbar = [sum(Q[h, i, c] for i in active) / len(active) for c in range(d)]
        logit = [sum(qbar[c] * K[h, j, c] for c in range(d)) / math.sqrt(d) for j in range(L)]
        z = sum(math.exp(x) for x in logit)
        for j in range(L):
            ref[j] += math.exp(logit[j]) / z / H
    assert np.allclose(S, ref, atol=1e-14)
    assert S.sum() == pytest.approx(1.0, abs=1e-12)
    # with a single active query the two readings coincide
    assert np.allclose(fo.sink_scores(Q, [2], K, pooled_query=True), fo.sink_scores(Q, [2], K), atol=1e-15)


# --------------------------------------------------------------------------- stage 3 (Eq. 8, Eq. 9)
def test_attention_index_set_membership():
    M, B = 23, 8
    got = fo.attention_index_set([3, 17, 22, 40, -1], [2, 0, -1], M, B)
    ref = [j for j in range(M) if j in (3, 17, 22) or j // B in (0, 2)]
    assert got.tolist() == ref
    # a sink inside a kept block, or listed twice, is still one element
    assert fo.attention_index_set([3, 3, 5], [0], M, B).tolist() == list(range(8))


def _sdpa(Q, K, V):
    t = lambda x: torch.from_numpy(np.ascontiguousarray(x))
    return torch.nn.functional.scaled_dot_product_attention(t(Q), t(K), t(V)).numpy()


def test_dense_reduction_equals_full_bidirectional_attention():
    # keep every block, take every row as a query: the sparse path must be plain softmax(QK^T/sqrt(d))V over all L keys
    H, M, N, d, B = 3, 37, 6, 16, 8
    Q, K, V = _rand(20, H, 11, d), _rand(21, H, M + N, d), _rand(22, H, M + N, d)
    n_b = -(-M // B)
    I_p = fo.attention_index_set([], np.arange(n_b), M, B)
    out, lse = fo.sparse_attention(Q, np.arange(11), K, V, I_p, M)
    assert np.allclose(out, _sdpa(Q, K, V), atol=1e-13)
    ref_lse = torch.logsumexp(torch.from_numpy(Q) @ torch.from_numpy(K).transpose(1, 2) / math.sqrt(d), dim=-1)
    assert np.allclose(lse, ref_lse.numpy(), atol=1e-13)
    # and through the per-layer driver with C = n_b
    r = fo.focus_layer(Q, K, V, [0, 1], np.arange(11), [5], M, B, n_b)
    assert np.allclose(r["out"], _sdpa(Q, K, V), atol=1e-13)


def test_sparse_attention_equals_attention_over_gathered_rows():
    H, M, N, d, B = 2, 40, 5, 8, 8
    Q, K, V = _rand(23, H, 9, d), _rand(24, H, M + N, d), _rand(25, H, M + N, d)
    I_p = fo.attention_index_set([1, 30], [2, 4], M, B)
    rows = [j for j in range(M + N) if j >= M or j in (1, 30) or j // B in (2, 4)]
    active = np.array([0, 4, 8])
    out, _ = fo.sparse_attention(Q, active, K, V, I_p, M)
    assert np.allclose(out, _sdpa(Q[:, active], K[:, rows], V[:, rows]), atol=1e-13)


def test_sparse_attention_closed_forms():
    H, M, N, d, B = 2, 16, 0, 4, 4
    Q, V = _rand(26, H, 3, d), _rand(27, H, M, d)
    K = np.tile(_rand(28, 1, 1, d), (H, M, 1))                # equal keys: output is the mean of the kept V rows
    I_p = fo.attention_index_set([9], [1], M, B)
    out, lse = fo.sparse_attention(Q, [0, 2], K, V, I_p, M)
    assert np.allclose(out, V[:, [4, 5, 6, 7, 9]].mean(axis=1, keepdims=True).repeat(2, axis=1), atol=1e-14)
    # a single kept key (no blocks, one sink, no response rows): the output is that V row exactly
    out1, _ = fo.sparse_attention(Q, [1], _rand(29, H, M, d), V, fo.attention_index_set([11], [], M, B), M)
    assert np.array_equal(out1[:, 0], V[:, 11])
    # one-hot: a huge logit on one key
    K2 = np.zeros((H, M, d)); K2[:, 6, 0] = 50.0
    Q2 = np.zeros((H, 1, d)); Q2[..., 0] = 50.0
    out2, _ = fo.sparse_attention(Q2, [0], K2, V, fo.attention_index_set([], [0, 1, 2], M, B), M)
    assert np.allclose(out2[:, 0], V[:, 6], atol=1e-12)


def test_sparse_attention_metamorphic():
    H, M, N, d, B = 3, 32, 4, 8, 8
    Q, K, V = _rand(30, H, 6, d), _rand(31, H, M + N, d), _rand(32, H, M + N, d)
    sinks, blocks, active = [2, 20], [1, 3], [0, 3, 5]
    I_p = fo.attention_index_set(sinks, blocks, M, B)
    out, lse = fo.sparse_attention(Q, active, K, V, I_p, M)
    assert np.array_equal(fo.sparse_attention(Q, active, K, 2 * V, I_p, M)[0], 2 * out)      # linear in V
    assert np.allclose(fo.sparse_attention(Q, active, K + _rand(33, 1, 1, d), V, I_p, M)[0], out, atol=1e-13)
    perm = [1, 2, 0]
    assert np.array_equal(fo.sparse_attention(Q[perm], active, K[perm], V[perm], I_p, M)[0], out[perm])
    assert np.array_equal(fo.attention_index_set(sinks[::-1], blocks[::-1], M, B), I_p)       # order of the sets
    assert np.array_equal(fo.attention_index_set(sinks + [9, 9, 2], blocks, M, B), I_p)       # dedupe (9 is in block 1)
    # softmax weights are a probability distribution: feeding V = 1 returns exactly-normalised rows
    ones, _ = fo.sparse_attention(Q, active, K, np.ones_like(V), I_p, M)
    assert np.allclose(ones, 1.0, atol=1e-14)


def test_key_shift_leaves_every_selection_unchanged():
    H, M, N, d, B = 4, 64, 8, 16, 8
    Q, K = _rand(34, H, 8, d), _rand(35, H, M + N, d)
    focus = [1, 2, 6]
    delta = _rand(36, 1, 1, d)
    R0 = fo.block_relevance(Q, focus, fo.block_means(K, M, B))
    R1 = fo.block_relevance(Q, focus, fo.block_means(K + delta, M, B))
    assert np.allclose(R1 - R0, (R1 - R0)[0], atol=1e-12)        # uniform shift of the scores
    assert fo.select_blocks(R0, 3).tolist() == fo.select_blocks(R1, 3).tolist()
    S0, S1 = fo.sink_scores(Q, focus, K), fo.sink_scores(Q, focus, K + delta)
    assert fo.select_sinks(S0, M, 3).tolist() == fo.select_sinks(S1, M, 3).tolist()


# --------------------------------------------------------------------------- step driver (Alg. 1): sink reuse
def test_step_reuses_probe_layer_sinks_unchanged():
    H, M, N, d, B, n_gen, n_layers = 2, 48, 8, 8, 8, 8, 5
    tensors = {l: (_rand(40 + l, H, n_gen, d), _rand(50 + l, H, M + N, d), _rand(60 + l, H, M + N, d))
               for l in range(n_layers)}
    conf = np.random.default_rng(70).random(n_gen).astype(np.float32)
    step = fo.focus_step(conf, None, 3, 0, 0, n_gen, lambda l: tensors[l], probe_layer=1, sparse_layers=[2, 3, 4],
                         n_ctx=M, block=B, n_keep=2, n_sink=3)
    Qp, Kp, _ = tensors[1]
    assert step["sinks"].tolist() == fo.select_sinks(fo.sink_scores(Qp, step["active"], Kp), M, 3).tolist()
    for l in (2, 3, 4):
        lay = step["layers"][l]
        assert lay["sinks_used"] is step["sinks"]                 # the same array object, not a recomputation
        Q, K, V = tensors[l]
        I_p = fo.attention_index_set(step["sinks"], lay["blocks"], M, B)
        assert np.array_equal(lay["out"], fo.sparse_attention(Q, step["active"], K, V, I_p, M)[0])
    # the sinks a deeper layer would find on its own differ, so reuse is not vacuous here
    own = [fo.select_sinks(fo.sink_scores(tensors[l][0], step["active"], tensors[l][1]), M, 3).tolist() for l in (2, 3, 4)]
    assert any(o != step["sinks"].tolist() for o in own)


def test_widen_bf16_exact():
    t = torch.tensor([1.0, -2.5, 0.333, 1e-30, 3e38, 0.0, -0.0], dtype=torch.bfloat16)
    bits = t.view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(fo.widen_bf16(bits), t.to(torch.float64).numpy())


# ----------------------------------------------------------------------------- Eq. 2 and Eq. 3
def test_token_confidence_against_torch_softmax_and_brute_force():
    rng = np.random.default_rng(71)
    x = rng.normal(0, 3, (6, 257))
    tok, conf = fo.token_confidence(x)
    p = torch.softmax(torch.from_numpy(x), dim=1)
    assert np.allclose(conf, p.max(dim=1).values.numpy(), rtol=1e-12)
    assert tok.tolist() == p.argmax(dim=1).tolist()            # no ties in continuous random data
    for i in range(6):                                          # and written out term by term
        z = [math.exp(v) for v in x[i]]
        assert conf[i] == pytest.approx(max(z) / sum(z), rel=1e-12)


def test_token_confidence_closed_forms():
    V = 1000
    tok, conf = fo.token_confidence(np.zeros((1, V)))
    assert tok.tolist() == [0] and conf[0] == pytest.approx(1.0 / V, rel=1e-14)       # uniform: 1/|V|, lowest id wins
    x = np.full((1, V), -3.0)
    x[0, [17, 400]] = 2.0                                                              # two equal maxima
    tok, conf = fo.token_confidence(x)
    assert tok.tolist() == [17]
    assert conf[0] == pytest.approx(1.0 / (2.0 + (V - 2) * math.exp(-5.0)), rel=1e-13)
    x = np.zeros((1, V))
    x[0, 123] = 80.0                                                                   # one dominant token
    tok, conf = fo.token_confidence(x)
    assert tok.tolist() == [123] and conf[0] == pytest.approx(1.0, abs=1e-30)
    x[0, 5] = -np.inf                                                                  # an excluded token changes nothing else
    assert fo.token_confidence(x)[1][0] == pytest.approx(1.0, abs=1e-30)


def test_token_confidence_invariances_and_mask():
    rng = np.random.default_rng(72)
    x = rng.normal(0, 2, (5, 300))
    tok, conf = fo.token_confidence(x)
    tok2, conf2 = fo.token_confidence(x + 11.5)                 # softmax ignores a common shift
    assert tok.tolist() == tok2.tolist() and np.allclose(conf, conf2, rtol=1e-12)
    perm = rng.permutation(300)
    tok3, conf3 = fo.token_confidence(x[:, perm])               # relabelling the vocabulary relabels the token
    assert np.allclose(conf, conf3, rtol=1e-12) and [int(perm[t]) for t in tok3] == tok.tolist()
    assert ((conf > 1.0 / 300) & (conf <= 1.0)).all()
    masked = np.array([1, 0, 1, 0, 0], dtype=np.uint8)
    tok4, conf4 = fo.token_confidence(x, masked)
    assert tok4.tolist() == [tok[0], -1, tok[2], -1, -1] and conf4.tolist() == [conf[0], 0.0, conf[2], 0.0, 0.0]
    # the confidences feed Eq. 4 directly
    assert fo.select_focus(conf4, masked, 1).tolist() == [0 if conf[0] >= conf[2] else 2]


def test_cache_update_touches_exactly_the_refreshed_rows():
    rng = np.random.default_rng(73)
    H, L, d, base = 3, 40, 8, 25
    Kc, Vc = rng.normal(size=(H, L, d)), rng.normal(size=(H, L, d))
    active = [1, 4, 5, 12]
    Kn, Vn = rng.normal(size=(H, 6, d)), rng.normal(size=(H, 6, d))      # two spare slots past the active list
    K2, V2 = fo.cache_update(Kc, Vc, Kn, Vn, active, base)
    for h in range(H):
        for r in range(L):
            if r - base in active:
                a = active.index(r - base)
                assert (K2[h, r] == Kn[h, a]).all() and (V2[h, r] == Vn[h, a]).all()
            else:
                assert (K2[h, r] == Kc[h, r]).all() and (V2[h, r] == Vc[h, r]).all()
    assert (Kc != K2).any() and K2 is not Kc                           # a copy; the inputs are untouched
    K3, V3 = fo.cache_update(K2, V2, Kn, Vn, active, base)             # idempotent
    assert (K3 == K2).all() and (V3 == V2).all()
    K4, _ = fo.cache_update(Kc, Vc, Kn, Vn, [], base)                  # U empty: pure reuse
    assert (K4 == Kc).all()


# ----------------------------------------------------------------------------- Alg. 1 across a block entry (decode_block)
def test_full_attention_equals_library_attention_and_a_loop():
    H, L, d = 2, 11, 4
    Q, K, V = _rand(81, H, 6, d), _rand(82, H, L, d), _rand(83, H, L, d)
    rows = [0, 2, 5]
    out, lse = fo.full_attention(Q, rows, K, V)
    tq, tk, tv = (torch.from_numpy(x) for x in (Q[:, rows], K, V))
    assert np.allclose(out, torch.nn.functional.scaled_dot_product_attention(tq, tk, tv).numpy(), atol=1e-13)
    assert np.allclose(lse, torch.logsumexp(tq @ tk.transpose(1, 2) / math.sqrt(d), dim=-1).numpy(), atol=1e-13)
    h, i = 1, 5                                                   # one row written out term by term
    w = [math.exp(sum(Q[h, i, c] * K[h, j, c] for c in range(d)) / math.sqrt(d)) for j in range(L)]
    ref = [sum(w[j] * V[h, j, c] for j in range(L)) / sum(w) for c in range(d)]
    assert np.allclose(out[h, 2], ref, atol=1e-13)


def _decode_case(seed=90, n_layers=5, l_dense=1, dense_tail=1, n_steps=2):
    H, M, N, d, B, n_gen = 2, 48, 8, 8, 8, 8
    L = M + N
    rng = np.random.default_rng(seed)
    ent = {l: tuple(rng.standard_normal((H, L, d)) for _ in range(3)) for l in range(n_layers)}
    steps = []
    masked = np.ones(n_gen, dtype=np.uint8)
    for t in range(n_steps):
        per_layer = {l: (rng.standard_normal((H, n_gen, d)), rng.standard_normal((H, n_gen, d)), rng.standard_normal((H, n_gen, d)))
                     for l in range(n_layers)}
        steps.append({"conf": rng.random(n_gen).astype(np.float32), "masked": masked.copy(), "k": 2,
                      "layer": (lambda pl: (lambda l: pl[l]))(per_layer), "_tensors": per_layer})
        masked[rng.integers(0, n_gen)] = 0                        # a position is unmasked between the steps
    kw = dict(n_layers=n_layers, l_dense=l_dense, dense_tail=dense_tail, n_ctx=M, row_base=M, block=B, window=2, lo=0, hi=n_gen,
              n_keep=2, n_sink=3)
    return ent, steps, kw, (H, M, N, d, B, n_gen)


def test_decode_block_entry_is_dense_bidirectional_attention_of_every_position():
    ent, steps, kw, (H, M, N, d, B, n_gen) = _decode_case()
    res = fo.decode_block(lambda l: ent[l], [], **kw)
    for l in range(kw["n_layers"]):
        tq, tk, tv = (torch.from_numpy(x) for x in ent[l])
        assert np.allclose(res["entry"][l], torch.nn.functional.scaled_dot_product_attention(tq, tk, tv).numpy(), atol=1e-12)
        assert np.array_equal(res["K_cache"][l], ent[l][1]) and np.array_equal(res["V_cache"][l], ent[l][2])   # U = every position


def test_decode_block_step_equals_a_from_scratch_step_on_the_updated_cache():
    """The last step of a block, replayed from nothing but the caches it left behind: the one-step driver (pinned on its
    own) on those caches must select the same sinks and blocks and give the same outputs."""
    ent, steps, kw, (H, M, N, d, B, n_gen) = _decode_case()
    res = fo.decode_block(lambda l: ent[l], steps, **kw)
    last, tens = res["steps"][-1], steps[-1]["_tensors"]
    n_layers, l_dense = kw["n_layers"], kw["l_dense"]
    sparse = [l for l in range(n_layers) if l_dense < l < n_layers - kw["dense_tail"]]
    assert sparse == [2, 3]
    ref = fo.focus_step(steps[-1]["conf"], steps[-1]["masked"], 2, kw["window"], 0, n_gen,
                        lambda l: (tens[l][0], res["K_cache"][l], res["V_cache"][l]), l_dense, sparse, M, B, kw["n_keep"], kw["n_sink"])
    assert last["focus"].tolist() == ref["focus"].tolist() and last["active"].tolist() == ref["active"].tolist()
    assert last["sinks"].tolist() == ref["sinks"].tolist() and np.array_equal(last["S"], ref["S"])
    for l in sparse:
        assert last["layers"][l]["kind"] == "sparse"
        assert last["layers"][l]["blocks"].tolist() == ref["layers"][l]["blocks"].tolist()
        assert np.array_equal(last["layers"][l]["out"], ref["layers"][l]["out"])
    for l in (0, 1, 4):                                          # dense prefix, probe layer, dense tail: every key attended
        assert last["layers"][l]["kind"] == "dense"
        tq = torch.from_numpy(tens[l][0][:, last["active"]])
        tk, tv = torch.from_numpy(res["K_cache"][l]), torch.from_numpy(res["V_cache"][l])
        assert np.allclose(last["layers"][l]["out"], torch.nn.functional.scaled_dot_product_attention(tq, tk, tv).numpy(), atol=1e-12)


def test_decode_block_cache_rows_persist_and_prompt_means_stay_frozen():
    ent, steps, kw, (H, M, N, d, B, n_gen) = _decode_case(seed=91, n_steps=3)
    res = fo.decode_block(lambda l: ent[l], steps, **kw)
    act = [r["active"].tolist() for r in res["steps"]]
    assert any(set(act[0]) - set(act[1]) - set(act[2]))          # some position is refreshed in step 1 only
    for l in range(kw["n_layers"]):                              # every layer, dense and sparse alike
        for pos in range(n_gen):
            row = M + pos
            writers = [t for t in range(3) if pos in act[t]]
            if not writers:                                      # never refreshed: the block-entry state (Eq. 3, reuse)
                assert np.array_equal(res["K_cache"][l][:, row], ent[l][1][:, row])
                assert np.array_equal(res["V_cache"][l][:, row], ent[l][2][:, row])
            else:                                                # the state of the LAST step that refreshed it
                t = writers[-1]
                a = act[t].index(pos)
                assert np.array_equal(res["K_cache"][l][:, row], steps[t]["_tensors"][l][1][:, a])
                assert np.array_equal(res["V_cache"][l][:, row], steps[t]["_tensors"][l][2][:, a])
        # prompt rows are never refreshed between block entries, so the representative keys formed at the entry stay valid
        assert np.array_equal(res["K_cache"][l][:, :M], ent[l][1][:, :M])
        assert np.array_equal(fo.block_means(res["K_cache"][l], M, B), fo.block_means(ent[l][1], M, B))


def test_decode_block_refreshed_positions_are_attended_with_their_new_states():
    """Eq. 3 by hand: one layer, one prompt row, one response row, zero queries and keys, so attention is the plain
    mean of the two value rows.  The refreshed response row must enter the step with its NEW value."""
    z = np.zeros((1, 2, 1))
    V_all = np.array([[[1.0], [2.0]]])
    step = {"conf": np.array([0.5], dtype=np.float32), "masked": None, "k": 1,
            "layer": lambda l: (np.zeros((1, 1, 1)), np.zeros((1, 1, 1)), np.array([[[10.0]]]))}
    res = fo.decode_block(lambda l: (z, z, V_all), [step], n_layers=1, l_dense=0, dense_tail=0, n_ctx=1, row_base=1, block=1,
                          window=0, lo=0, hi=1, n_keep=1, n_sink=1)
    assert res["entry"][0][0, :, 0].tolist() == [1.5, 1.5]
    assert res["steps"][0]["layers"][0]["out"][0, 0, 0] == pytest.approx(5.5, abs=1e-15)     # (1 + 10) / 2, not (1 + 2) / 2
    assert res["V_cache"][0][0, :, 0].tolist() == [1.0, 10.0]
    assert res["steps"][0]["sinks"].tolist() == [0]
