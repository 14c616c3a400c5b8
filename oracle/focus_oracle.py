"""CPU oracle for the Focus-dLLM sparse-attention step.  TEST INFRASTRUCTURE ONLY.

This is the slow, plain reference the GPU library is checked against.  Only tests, the smoke
check and the benchmark's CPU-baseline leg may import it; the product never does.  It shares
no code with the HIP sources.

Every function follows one passage of the paper (Focus-dLLM, arXiv 2602.02159), cited in its
docstring, in the paper's order and notation.  All arithmetic is float64; bf16 / fp32 inputs
are widened exactly first.  numpy's matmul and sort are the only library steps.

Notation: H heads, d head_dim, M prompt (context) tokens, N response rows stored after the
prompt in K/V, L = M + N, B prompt block size, n_b = ceil(M / B).
Layouts: Q [H, n_gen, d], K and V [H, L, d].

Readings taken where the paper leaves a choice (each restated where it is used):
  * every top-k orders by (value descending, index ascending); -0.0 == +0.0; NaN ranks last;
    index sets are returned ascending;
  * I_focus has min(k, #masked) entries; the window is clipped to a caller range [lo, hi);
  * the queries of I_focus enter the block relevance through their mean (no 1/sqrt(d));
  * the sink score is the column mass of that layer's attention: softmax per (head, active
    query) over all L keys, then the mean over heads and active queries; only prompt
    positions are sink candidates;
  * the last prompt block may be shorter than B and is averaged over its true length;
  * the key set of the sparse attention is a set: a sink inside a kept block counts once;
  * the arg max of Eq. 2 goes to the lower token id when several tokens share the maximum;
  * Eq. 3 defines the keys a step USES: the refreshed positions enter that step's attention with their
    newly computed states.  Alg. 1 prints the cache update after the attention and only in its dense
    branch; here every layer (dense or sparse) first writes the new states of I_active into its cache
    and then attends over the cache.

Pins (tests/test_oracle_*.py): dense reduction against an independent attention, softmax row
sums, brute-force top-k, closed forms (equal keys, single key, one-hot), linearity of the
block relevance, metamorphic invariances.  No function here is "parity unpinned"; the paper
prints no numeric example of this path, so absolute values are pinned through those
identities rather than through printed numbers.
"""
from __future__ import annotations

import math

import numpy as np

__all__ = [
    "widen_bf16", "top_indices", "decision_margin", "select_focus", "expand_window", "block_means",
    "block_relevance", "select_blocks", "sink_scores", "select_sinks", "attention_index_set",
    "sparse_attention", "focus_layer", "focus_step", "token_confidence", "cache_update", "full_attention",
    "decode_block",
]


# ----------------------------------------------------------------------------- helpers
def widen_bf16(bits) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float64, exactly (bf16 is the top half of an fp32)."""
    b = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


def _f64(x) -> np.ndarray:
    return np.asarray(x, dtype=np.float64)


def top_indices(values, n: int, candidates=None) -> np.ndarray:
    """Indices of the n best entries under the total order (value desc, index asc), ascending.

    NaN ranks below every number and -0.0 equals +0.0.  `candidates` (bool mask or None)
    restricts the ranking; fewer than n candidates returns them all.
    """
    v = _f64(values).ravel() + 0.0  # +0.0 folds -0.0 into +0.0
    idx = np.arange(v.size)
    if candidates is not None:
        idx = idx[np.asarray(candidates, dtype=bool).ravel()]
    vv = v[idx]
    nan = np.isnan(vv)
    neg = np.where(nan, 0.0, -vv)
    order = np.lexsort((idx, neg, nan))  # primary: non-NaN first; then larger value; then lower index
    return np.sort(idx[order[: max(0, min(n, idx.size))]]).astype(np.int64)


def decision_margin(values, n: int, candidates=None) -> float:
    """Gap between the last kept and the first dropped value of a top-n, relative to the value spread.

    inf when nothing is dropped or kept.  Used to make "bit-exact indices" well posed: a workload is
    admissible for index parity only if this exceeds the fp32 reordering noise by a wide factor.
    """
    v = _f64(values).ravel()
    if candidates is not None:
        v = v[np.asarray(candidates, dtype=bool).ravel()]
    v = np.sort(v[~np.isnan(v)])[::-1]
    if n <= 0 or n >= v.size:
        return math.inf
    spread = v[0] - v[-1]
    return math.inf if spread == 0 else float((v[n - 1] - v[n]) / spread)


# ----------------------------------------------------------------------------- stage 1
def select_focus(conf, masked, k: int) -> np.ndarray:
    """I_focus (Sec. 5.2, Eq. 4): the k still-masked positions of the current block with the highest
    previous-step confidence.  Reading: min(k, #masked) entries; ties to the lower position."""
    conf = _f64(conf)
    m = np.ones(conf.shape, bool) if masked is None else np.asarray(masked).astype(bool)
    return top_indices(conf, k, m)


def expand_window(focus, w: int, lo: int, hi: int) -> np.ndarray:
    """I_active (Sec. 5.2, Eq. 5): union over i in I_focus of {l : i - floor(w/2) <= l <= i + floor(w/2)},
    clipped to [lo, hi) (reading: the caller's valid query rows), ascending without repeats."""
    half = int(w) // 2
    s = set()
    for i in np.asarray(focus, dtype=np.int64).tolist():
        for l in range(i - half, i + half + 1):
            if lo <= l < hi:
                s.add(l)
    return np.array(sorted(s), dtype=np.int64)


# ----------------------------------------------------------------------------- stage 2a
def block_means(K, n_ctx: int, block: int) -> np.ndarray:
    """Representative keys (Sec. 5.3, "Block-wise token pruning"): K_bar[h, b] = mean of K[h, j] over the
    prompt rows j of block b = [b*B, min((b+1)*B, M)).  Returns [H, n_b, d]."""
    H, _, d = K.shape
    n_b = -(-n_ctx // block)
    out = np.empty((H, n_b, d), dtype=np.float64)
    for h in range(H):
        Kh = _f64(K[h, :n_ctx])
        for b in range(n_b):
            out[h, b] = Kh[b * block: min((b + 1) * block, n_ctx)].mean(axis=0)
    return out


def block_relevance(Q, focus, kbar) -> np.ndarray:
    """R_b (Sec. 5.3, Eq. 7) = (1/H) sum_h Q^h_{I_focus} . K_bar^h_b.  Reading: the focus queries are
    aggregated by their mean, and no 1/sqrt(d) is applied (neither changes the ranking)."""
    focus = np.asarray(focus, dtype=np.int64)
    H = Q.shape[0]
    R = np.zeros(kbar.shape[1], dtype=np.float64)
    for h in range(H):
        q_bar = _f64(Q[h])[focus].mean(axis=0)
        R += kbar[h] @ q_bar
    return R / H


def select_blocks(R, n_keep: int) -> np.ndarray:
    """B_relevant = Top-C(R_b) (Sec. 5.3), ascending block ids; C is passed as an integer."""
    return top_indices(R, n_keep)


# ----------------------------------------------------------------------------- stage 2b
def sink_scores(Q, active, K, pooled_query: bool = False) -> np.ndarray:
    """S_j (Sec. 5.3, Eq. 6) for every key j in [0, L).

    Default reading (column mass): P[h, i, :] = softmax over all L keys of Q[h, i] . K[h, j] / sqrt(d) for
    each active query i, and S_j is the mean of P[h, i, j] over heads and active queries.
    pooled_query=True is the other reading of the text (mean the active queries first, then one
    softmax per head); kept only so the two can be compared.
    """
    active = np.asarray(active, dtype=np.int64)
    H, L, d = K.shape
    S = np.zeros(L, dtype=np.float64)
    for h in range(H):
        q = _f64(Q[h])[active]
        if pooled_query:
            q = q.mean(axis=0, keepdims=True)
        logits = (q @ _f64(K[h]).T) / math.sqrt(d)
        logits -= logits.max(axis=1, keepdims=True)
        p = np.exp(logits)
        p /= p.sum(axis=1, keepdims=True)
        S += p.mean(axis=0)
    return S / H


def select_sinks(S, n_ctx: int, n_sink: int) -> np.ndarray:
    """I_sink = Top-N_sink(S_j) (Sec. 5.3).  Reading: only prompt positions j < M are candidates (response
    rows are always attended anyway)."""
    cand = np.zeros(len(S), bool)
    cand[:n_ctx] = True
    return top_indices(S, n_sink, cand)


# ----------------------------------------------------------------------------- stage 3
def attention_index_set(sinks, blocks, n_ctx: int, block: int) -> np.ndarray:
    """I_p (Sec. 5.3, Eq. 8): the sinks united with every prompt position of every kept block, as a set,
    ascending.  Entries outside the prompt (negative padding included) are ignored."""
    s = set(int(j) for j in np.asarray(sinks, dtype=np.int64).tolist() if 0 <= j < n_ctx)
    n_b = -(-n_ctx // block)
    for b in np.asarray(blocks, dtype=np.int64).tolist():
        if 0 <= b < n_b:
            s.update(range(b * block, min((b + 1) * block, n_ctx)))
    return np.array(sorted(s), dtype=np.int64)


def sparse_attention(Q, active, K, V, index_set, n_ctx: int):
    """Attn (Sec. 5.3, Eq. 9): softmax(Q_active K_attn^T / sqrt(d)) V_attn with K_attn = concat(K[I_p],
    K_resp), likewise V; bidirectional, no mask.  Returns (out [H, n_q, d], lse [H, n_q]) in float64,
    lse being the natural-log sum of exp of the scaled logits."""
    active = np.asarray(active, dtype=np.int64)
    H, L, d = K.shape
    J = np.concatenate([np.asarray(index_set, dtype=np.int64), np.arange(n_ctx, L, dtype=np.int64)])
    out = np.empty((H, len(active), d), dtype=np.float64)
    lse = np.empty((H, len(active)), dtype=np.float64)
    for h in range(H):
        q = _f64(Q[h])[active]
        logits = (q @ _f64(K[h][J]).T) / math.sqrt(d)
        m = logits.max(axis=1, keepdims=True)
        p = np.exp(logits - m)
        z = p.sum(axis=1, keepdims=True)
        out[h] = (p / z) @ _f64(V[h][J])
        lse[h] = (m + np.log(z))[:, 0]
    return out, lse


# ----------------------------------------------------------------------------- per layer / per step
def focus_layer(Q, K, V, focus, active, sinks, n_ctx: int, block: int, n_keep: int) -> dict:
    """One sparse layer (Alg. 1, the branch taken when sparse attention is on and l > l_dense)."""
    kbar = block_means(K, n_ctx, block)
    R = block_relevance(Q, focus, kbar)
    blocks = select_blocks(R, n_keep)
    I_p = attention_index_set(sinks, blocks, n_ctx, block)
    out, lse = sparse_attention(Q, active, K, V, I_p, n_ctx)
    return {"kbar": kbar, "R": R, "blocks": blocks, "index_set": I_p, "out": out, "lse": lse}


def focus_step(conf, masked, k: int, w: int, lo: int, hi: int, layers, probe_layer: int, sparse_layers,
               n_ctx: int, block: int, n_keep: int, n_sink: int) -> dict:
    """One non-block-entry denoising step over a stack of layers (Alg. 1): queries are selected once
    before the layer loop; the sinks are identified once, from the probe layer's attention, and the
    same index array is handed unchanged to every sparse layer.  `layers(l)` returns that layer's (Q, K, V)."""
    focus = select_focus(conf, masked, k)
    active = expand_window(focus, w, lo, hi)
    Qp, Kp, _ = layers(probe_layer)
    S = sink_scores(Qp, active, Kp)
    sinks = select_sinks(S, n_ctx, n_sink)
    per_layer = {}
    for l in sparse_layers:
        Q, K, V = layers(l)
        per_layer[l] = focus_layer(Q, K, V, focus, active, sinks, n_ctx, block, n_keep)
        per_layer[l]["sinks_used"] = sinks  # the identical object on purpose
    return {"focus": focus, "active": active, "S": S, "sinks": sinks, "layers": per_layer}


# ----------------------------------------------------------------------------- around the step (Sec. 3)
def token_confidence(logits, masked=None):
    """Predicted token and confidence of every position (Eq. 2).

    p(x_i = v) is the softmax of row i of `logits` [n, |V|] over the vocabulary;
    x_hat_i = argmax_v p(x_i = v) and c_i = max_v p(x_i = v) = 1 / sum_v exp(logit_iv - max_v logit_iv).
    The paper does not say which token wins a tie of the maximum: the lower id does.  Positions with
    masked[i] == 0 are no candidates of Eq. 4; they get token -1 and confidence 0.
    Returns (tokens int64 [n], conf float64 [n]).
    """
    x = _f64(logits)
    n, _ = x.shape
    tokens = np.full(n, -1, dtype=np.int64)
    conf = np.zeros(n, dtype=np.float64)
    for i in range(n):
        if masked is not None and not masked[i]:
            continue
        row = x[i]
        m = row.max()
        tokens[i] = int(np.flatnonzero(row == m)[0])
        conf[i] = 1.0 / np.exp(row - m).sum()
    return tokens, conf


def cache_update(K_cache, V_cache, K_new, V_new, active, row_base: int):
    """Approximate KV cache (Eq. 3): the refreshed set U = {row_base + i : i in I_active} takes the newly
    computed states, every other row keeps its cached one.

    K_cache, V_cache [H, L, d]; K_new, V_new [H, >= |I_active|, d] hold the new states of the active positions in
    list order; `row_base` is the cache row of position 0 of the generation block.  Returns new arrays.
    """
    K_out, V_out = np.array(K_cache, copy=True), np.array(V_cache, copy=True)
    for a, i in enumerate(np.asarray(active, dtype=np.int64).tolist()):
        K_out[:, row_base + i, :] = K_new[:, a, :]
        V_out[:, row_base + i, :] = V_new[:, a, :]
    return K_out, V_out


# ----------------------------------------------------------------------------- Alg. 1 across a block entry
def full_attention(Q, rows, K, V):
    """FullAttn of Alg. 1: softmax(Q_rows K^T / sqrt(d)) V over every row of K / V, bidirectional.
    Returns (out [H, len(rows), d], lse [H, len(rows)]) in float64."""
    rows = np.asarray(rows, dtype=np.int64)
    H, L, d = K.shape
    out = np.empty((H, len(rows), d), dtype=np.float64)
    lse = np.empty((H, len(rows)), dtype=np.float64)
    for h in range(H):
        logits = (_f64(Q[h])[rows] @ _f64(K[h]).T) / math.sqrt(d)
        m = logits.max(axis=1, keepdims=True)
        p = np.exp(logits - m)
        z = p.sum(axis=1, keepdims=True)
        out[h] = (p / z) @ _f64(V[h])
        lse[h] = (m + np.log(z))[:, 0]
    return out, lse


def decode_block(entry, steps, n_layers: int, l_dense: int, dense_tail: int, n_ctx: int, row_base: int, block: int,
                 window: int, lo: int, hi: int, n_keep: int, n_sink: int) -> dict:
    """Alg. 1 for one generation block over a stack of attention layers with an approximate KV cache (Sec. 3,
    Eq. 3): the block-entry step, then the sparse steps that follow it.

    Layers are numbered from 0; layers 0 .. l_dense attend densely, layer l_dense is the one whose attention
    identifies the sinks, the last `dense_tail` layers stay dense as well, every layer in between is sparse.

    entry(l) -> (Q_all, K_all, V_all), each [H, L, d]: the states of EVERY position as computed at the block entry
        (I_active = all positions, no pruning): the whole cache of layer l is rewritten (Eq. 3 with U = everything)
        and every position attends to every key.
    steps: a list, one dict per later step, with
        'conf' [n_gen], 'masked' [n_gen] or None, 'k'  -> I_focus (Eq. 4) and I_active (Eq. 5, window / lo / hi);
        'layer': l -> (Q [H, n_gen, d], K_new [H, >= |I_active|, d], V_new): the queries of the generation block and
        the newly computed states of the active positions in list order.
      In every layer the cache rows row_base + i, i in I_active, first take the new states (Eq. 3); then
        a dense layer attends with Q[I_active] over the whole cache; at l_dense S_j (Eq. 6) is read off that
        attention and I_sink selected; a sparse layer runs Eq. 7, Top-C, Eq. 8 and Eq. 9 on the cache with those sinks.
    Returns {'entry': [out_l [H, L, d]], 'steps': [{'focus', 'active', 'S', 'sinks', 'layers': [..per layer dict..]}],
             'K_cache': [..], 'V_cache': [..]} (caches after the last step).
    """
    K_cache, V_cache, entry_out = [], [], []
    for l in range(n_layers):
        Q_all, K_all, V_all = entry(l)
        L = K_all.shape[1]
        K_cache.append(np.array(K_all, dtype=np.float64, copy=True))
        V_cache.append(np.array(V_all, dtype=np.float64, copy=True))
        entry_out.append(full_attention(Q_all, np.arange(L), K_cache[l], V_cache[l])[0])
    first_tail = n_layers - dense_tail
    results = []
    for st in steps:
        focus = select_focus(st["conf"], st.get("masked"), st["k"])
        active = expand_window(focus, window, lo, hi)
        sinks, S, per_layer = None, None, []
        for l in range(n_layers):
            Q, K_new, V_new = st["layer"](l)
            K_cache[l], V_cache[l] = cache_update(K_cache[l], V_cache[l], _f64(K_new), _f64(V_new), active, row_base)
            if l <= l_dense or l >= first_tail:
                out, lse = full_attention(Q, active, K_cache[l], V_cache[l])
                rec = {"kind": "dense", "out": out, "lse": lse}
                if l == l_dense:
                    S = sink_scores(Q, active, K_cache[l])
                    sinks = select_sinks(S, n_ctx, n_sink)
            else:
                rec = focus_layer(Q, K_cache[l], V_cache[l], focus, active, sinks, n_ctx, block, n_keep)
                rec["kind"] = "sparse"
            per_layer.append(rec)
        results.append({"focus": focus, "active": active, "S": S, "sinks": sinks, "layers": per_layer})
    return {"entry": entry_out, "steps": results, "K_cache": K_cache, "V_cache": V_cache}
