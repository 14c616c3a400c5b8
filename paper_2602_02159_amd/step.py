"""Sequencing of the C-ABI calls for one denoising step over a stack of layers (Alg. 1 of the paper).

Nothing is computed here: the class owns the device buffers (index sets, scores, outputs, workspaces),
marshals every call's arguments once, and `run` enqueues the library calls in the order the algorithm
prescribes, all on the current stream, with no host synchronisation between them — the index sets produced
by one call are consumed on the device by the next.  Because a step is a fixed sequence of launches on
fixed buffers it can also be captured into a HIP graph (`capture`) and replayed.

FocusStep runs one step over layers whose K/V tensors are given; FocusDecoder owns the KV caches and sequences a
whole generation block: the block entry, then steps with the per-layer cache updates of Eq. 3.
"""
from __future__ import annotations

import ctypes as C

import torch

from . import binding as fb


class FocusStep:
    """Buffers and call sequence for one step.

    Layers are (q, k, v) bf16 CUDA tensors in [H, rows, d] layout: q [H, n_gen, d]; k, v [H, M+N, d].
    `probe` is the (q, k) pair of the layer whose attention identifies the sinks, or its (q, k, v) triple: then the
    stage "probe_layer" (that layer's dense attention and the sinks in one call) is available as well and, with
    `use_probe_layer`, replaces "find_sinks" in the step.
    `logits` (bf16 [n_gen, vocab], optional): the step then starts with focus_token_confidence, whose output is the
    confidence the query selection ranks (`conf` is overwritten).
    `dense_tail`: the last so many layers attend to every block (the schedule that keeps the final layers dense).
    `kbars` (optional, one fp32 [H, n_b, d] tensor per layer): block means the caller already holds — what
    focus_cache_refresh emitted at the block entry — used by the cached-means stages instead of buffers of this object.
    """

    def __init__(self, conf, masked, probe, sparse_layers, n_ctx: int, block: int, k_focus: int, window: int, n_keep: int,
                 n_sink: int, cached_means: bool = False, dense: bool = False, logits=None, dense_tail: int = 0, kbars=None):
        q0 = probe[0]
        dev = q0.device
        self.H, self.n_gen, self.d = q0.shape
        self.M, self.B = n_ctx, block
        self.n_b = -(-n_ctx // block)
        self.k_focus, self.window, self.n_keep, self.n_sink = k_focus, window, n_keep, n_sink
        self.max_active = min(self.n_gen, k_focus * (2 * (window // 2) + 1))
        i32 = lambda n: torch.full((max(n, 1),), -1, dtype=torch.int32, device=dev)
        self.focus_idx, self.active_idx, self.counts, self.sink_idx = i32(k_focus), i32(self.max_active), i32(2), i32(n_sink)
        self.col_mass = torch.empty(probe[1].shape[1], dtype=torch.float32, device=dev)
        self.all_blocks = torch.arange(self.n_b, dtype=torch.int32, device=dev)
        self.conf, self.masked, self.probe, self.layers = conf, masked, probe, list(sparse_layers)
        self.dense_tail, self.use_probe_layer = dense_tail, False
        self.tokens = i32(self.n_gen)
        self.bufs = [{
            "kept": i32(n_keep),
            "scores": torch.empty(self.n_b, dtype=torch.float32, device=dev),
            "out": torch.zeros((self.H, self.max_active, self.d), dtype=torch.bfloat16, device=dev),
            "kbar": kbars[i] if kbars is not None else torch.empty((self.H, self.n_b, self.d), dtype=torch.float32, device=dev),
            "partials": torch.empty((self.H, self.n_b), dtype=torch.float32, device=dev),
        } for i in range(len(self.layers))]
        self._keep = []  # shapes and workspaces referenced by raw pointers below
        L = fb.lib()
        p = lambda t: None if t is None else C.c_void_p(t.data_ptr())

        def workspace(nbytes):
            t = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
            self._keep.append(t)
            return t

        s_probe = fb.make_shape(probe[0], probe[1], None, n_ctx, block)
        self._keep.append(s_probe)
        ws_sinks = workspace(fb.workspace_bytes(fb.FN_FIND_SINKS, s_probe, self.max_active))
        self.calls = {
            "select": [(L.focus_select_queries, (p(conf), p(masked), self.n_gen, k_focus, window, 0, self.n_gen,
                                                 p(self.focus_idx), p(self.active_idx), self.max_active, p(self.counts)))],
            "find_sinks": [(L.focus_find_sinks, (p(probe[0]), p(self.active_idx), p(self.counts), self.max_active, p(probe[1]),
                                                 C.byref(s_probe), n_sink, p(self.col_mass), p(self.sink_idx), p(ws_sinks),
                                                 ws_sinks.numel()))],
            "block_means": [], "block_scores": [], "block_scores_cached": [], "sparse_attn": [], "dense_attn": [],
            "sparse_layer": [], "sparse_layer_cached": [], "block_partials": [], "probe_layer": [],
        }
        if len(probe) == 3:
            self.probe_out = torch.zeros((self.H, self.max_active, self.d), dtype=torch.bfloat16, device=dev)
            s_pl = fb.make_shape(probe[0], probe[1], probe[2], n_ctx, block, self.probe_out)
            self._keep.append(s_pl)
            ws_pl = workspace(fb.workspace_bytes(fb.FN_PROBE_LAYER, s_pl, self.max_active))
            self.calls["probe_layer"] = [(L.focus_probe_layer, (
                p(probe[0]), p(self.active_idx), p(self.counts), self.max_active, p(probe[1]), p(probe[2]), C.byref(s_pl),
                n_sink, p(self.probe_out), None, p(self.col_mass), p(self.sink_idx), p(ws_pl), ws_pl.numel()))]
        ws_scores = ws_attn = ws_dense = ws_layer = None
        for (q, k, v), b in zip(self.layers, self.bufs):
            s = fb.make_shape(q, k, v, n_ctx, block, b["out"])
            self._keep.append(s)
            sp = C.byref(s)
            if ws_scores is None:
                ws_scores = workspace(fb.workspace_bytes(fb.FN_BLOCK_SCORES, s))
                ws_attn = workspace(fb.workspace_bytes(fb.FN_SPARSE_ATTN, s, self.max_active, n_keep, n_sink))
                ws_dense = workspace(fb.workspace_bytes(fb.FN_SPARSE_ATTN, s, self.max_active, self.n_b, 0))
                ws_layer = workspace(fb.workspace_bytes(fb.FN_SPARSE_LAYER, s, self.max_active, n_keep, n_sink))
            self.calls["block_means"].append((L.focus_block_means, (p(k), sp, p(b["kbar"]))))
            self.calls["block_partials"].append((L.focus_block_partials, (
                p(q), p(self.focus_idx), p(self.counts), k_focus, p(k), None, sp, p(b["partials"]))))
            self.calls["block_scores"].append((L.focus_block_scores, (
                p(q), p(self.focus_idx), p(self.counts), k_focus, p(k), None, sp, n_keep, p(b["scores"]), p(b["kept"]),
                p(ws_scores), ws_scores.numel())))
            self.calls["block_scores_cached"].append((L.focus_block_scores, (
                p(q), p(self.focus_idx), p(self.counts), k_focus, None, p(b["kbar"]), sp, n_keep, p(b["scores"]), p(b["kept"]),
                p(ws_scores), ws_scores.numel())))
            self.calls["sparse_attn"].append((L.focus_sparse_attn, (
                p(q), p(self.active_idx), p(self.counts), self.max_active, p(k), p(v), sp, p(b["kept"]), n_keep,
                p(self.sink_idx), n_sink, p(b["out"]), None, p(ws_attn), ws_attn.numel())))
            for stage, kb in (("sparse_layer", None), ("sparse_layer_cached", p(b["kbar"]))):
                self.calls[stage].append((L.focus_sparse_layer, (
                    p(q), p(self.focus_idx), p(self.active_idx), p(self.counts), k_focus, self.max_active, p(k), p(v), kb, sp,
                    n_keep, p(self.sink_idx), n_sink, p(b["scores"]), p(b["kept"]), p(b["out"]), None, p(ws_layer),
                    ws_layer.numel())))
            self.calls["dense_attn"].append((L.focus_sparse_attn, (
                p(q), p(self.active_idx), p(self.counts), self.max_active, p(k), p(v), sp, p(self.all_blocks), self.n_b,
                None, 0, p(b["out"]), None, p(ws_dense), ws_dense.numel())))
        self.calls["confidence"] = []
        if logits is not None:
            ws_conf = workspace(fb.token_confidence_workspace(logits.shape[0], logits.shape[1]))
            self.calls["confidence"] = [(L.focus_token_confidence, (
                p(logits), logits.stride(0), p(masked), logits.shape[0], logits.shape[1], p(self.tokens), p(conf), p(ws_conf),
                ws_conf.numel()))]
            self._keep.append(logits)
        self.cached_means, self.dense, self.fused = cached_means, dense, True
        self._graph = None

    @staticmethod
    def _issue(calls, stream):
        for fn, args in calls:
            rc = fn(*args, stream)
            if rc != 0:
                raise fb.FocusError(rc, fb.last_error())

    def issue(self, stage: str, layer: int | None = None):
        """Enqueue one stage (all layers, or one) on the current stream."""
        calls = self.calls[stage]
        self._issue(calls if layer is None else calls[layer:layer + 1], torch.cuda.current_stream().cuda_stream)

    def sequence(self):
        """The step's calls in order: [confidence,] queries once, sinks once at the probe layer, then every layer."""
        seq = self.calls["confidence"] + self.calls["select"]
        seq = seq + (self.calls["probe_layer"] if self.use_probe_layer and self.calls["probe_layer"] else self.calls["find_sinks"])
        if self.dense:
            return seq + self.calls["dense_attn"]
        n = len(self.layers)
        first_dense = n - min(self.dense_tail, n)
        if self.fused:  # one call per sparse layer: block scores and attention in three launches
            per_layer = self.calls["sparse_layer_cached" if self.cached_means else "sparse_layer"]
            return seq + per_layer[:first_dense] + self.calls["dense_attn"][first_dense:]
        scores = self.calls["block_scores_cached" if self.cached_means else "block_scores"]
        for i in range(first_dense):
            seq = seq + [scores[i], self.calls["sparse_attn"][i]]
        return seq + self.calls["dense_attn"][first_dense:]

    def run(self):
        """Enqueue one whole step (eagerly, or by replaying the captured graph)."""
        if self._graph is not None:
            self._graph.replay()
        else:
            self._issue(self.sequence(), torch.cuda.current_stream().cuda_stream)

    def capture(self):
        """Capture the step into a HIP graph; later `run` calls replay it."""
        self._graph = None
        self.run()  # warm: module loading must not happen under capture
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            self._issue(self.sequence(), torch.cuda.current_stream().cuda_stream)
        self._graph = g

    def release_graph(self):
        self._graph = None


class FocusDecoder:
    """Alg. 1 of the paper for one generation block over a stack of attention layers with an approximate KV cache:
    the block-entry step (every position recomputed, caches rewritten, block means formed) and the sparse steps after
    it, each as a fixed sequence of C-ABI calls on fixed buffers that can be replayed as a HIP graph.

    Layers are numbered from 0: layers 0 .. l_dense attend densely (l_dense is the probe layer, whose attention also
    yields the sinks), the last `dense_tail` layers stay dense, the layers in between are sparse.  Nothing is computed
    here; the caller (a model's projections; in the tests a random generator) fills the input buffers:

      block entry   q_all[l], k_all[l], v_all[l]   bf16 [H, M+N, d]      states of every position
      step          conf fp32 [n_gen] (or logits), masked u8 [n_gen],
                    q[l] bf16 [H, n_gen, d], k_new[l] / v_new[l] bf16 [H, max_active, d]: slot a = position I_active[a]

    run_entry():  per layer  focus_cache_refresh (cache rows <- new states, K_bar of the sparse layers from the same pass),
                  focus_refresh_attn (every position attends to every key)            -> out_all[l]
    run_step():   [focus_token_confidence,] focus_select_queries, then per layer focus_cache_update (Eq. 3: the active rows
                  take their new states before the layer attends) followed by
                    dense layer   focus_sparse_attn with every block kept
                    probe layer   focus_probe_layer (dense attention + I_sink)
                    sparse layer  focus_sparse_layer with the K_bar cached at the block entry -> out[l], kept[l], scores[l]
    `row_base` is the cache row of position 0 of the generation block.
    """

    def __init__(self, n_layers: int, l_dense: int, dense_tail: int, n_heads: int, head_dim: int, n_ctx: int, n_resp: int,
                 n_gen: int, row_base: int, block: int, k_focus: int, window: int, n_keep: int, n_sink: int, device,
                 vocab: int | None = None):
        assert 0 <= l_dense < n_layers and 0 <= dense_tail <= n_layers - l_dense - 1
        self.n_layers, self.l_dense, self.first_tail = n_layers, l_dense, n_layers - dense_tail
        H, d, L = n_heads, head_dim, n_ctx + n_resp
        self.H, self.d, self.M, self.L, self.B, self.n_gen = H, d, n_ctx, L, block, n_gen
        self.n_b = -(-n_ctx // block)
        self.max_active = min(n_gen, k_focus * (2 * (window // 2) + 1))
        dev = device
        bf = lambda *shape: torch.zeros(shape, dtype=torch.bfloat16, device=dev)
        i32 = lambda n: torch.full((max(n, 1),), -1, dtype=torch.int32, device=dev)
        self.k_cache = [bf(H, L, d) for _ in range(n_layers)]
        self.v_cache = [bf(H, L, d) for _ in range(n_layers)]
        self.kbar = [torch.zeros((H, self.n_b, d), dtype=torch.float32, device=dev) if self.is_sparse(l) else None
                     for l in range(n_layers)]
        self.q_all, self.k_all, self.v_all = ([bf(H, L, d) for _ in range(n_layers)] for _ in range(3))
        self.out_all = [bf(H, L, d) for _ in range(n_layers)]
        self.conf = torch.zeros(n_gen, dtype=torch.float32, device=dev)
        self.masked = torch.ones(n_gen, dtype=torch.uint8, device=dev)
        self.logits = None if vocab is None else torch.zeros((n_gen, vocab), dtype=torch.bfloat16, device=dev)
        self.tokens = i32(n_gen)
        self.q = [bf(H, n_gen, d) for _ in range(n_layers)]
        self.k_new = [bf(H, self.max_active, d) for _ in range(n_layers)]
        self.v_new = [bf(H, self.max_active, d) for _ in range(n_layers)]
        self.out = [bf(H, self.max_active, d) for _ in range(n_layers)]
        self.kept = [i32(n_keep) for _ in range(n_layers)]
        self.scores = [torch.zeros(self.n_b, dtype=torch.float32, device=dev) for _ in range(n_layers)]
        self.focus_idx, self.active_idx, self.counts, self.sink_idx = i32(k_focus), i32(self.max_active), i32(2), i32(n_sink)
        self.col_mass = torch.zeros(L, dtype=torch.float32, device=dev)
        self.all_blocks = torch.arange(self.n_b, dtype=torch.int32, device=dev)
        self._keep = []
        lib = fb.lib()
        p = lambda t: None if t is None else C.c_void_p(t.data_ptr())

        def workspace(nbytes):
            t = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
            self._keep.append(t)
            return t

        def shape(q, k, v, out=None):
            s = fb.make_shape(q, k, v, n_ctx, block, out)
            self._keep.append(s)
            return s

        self.entry_calls, self.step_calls = [], []
        for l in range(n_layers):
            s_all = shape(self.q_all[l], self.k_cache[l], self.v_cache[l], self.out_all[l])
            self.entry_calls.append((lib.focus_cache_refresh, (
                p(self.k_cache[l]), p(self.v_cache[l]), C.byref(s_all), p(self.k_all[l]), p(self.v_all[l]),
                self.k_all[l].stride(0), self.k_all[l].stride(1), p(self.kbar[l]))))
            self.entry_calls.append((lib.focus_refresh_attn, (
                p(self.q_all[l]), p(self.k_cache[l]), p(self.v_cache[l]), C.byref(s_all), p(self.out_all[l]), None)))
        if self.logits is not None:
            ws_conf = workspace(fb.token_confidence_workspace(n_gen, vocab))
            self.step_calls.append((lib.focus_token_confidence, (
                p(self.logits), self.logits.stride(0), p(self.masked), n_gen, vocab, p(self.tokens), p(self.conf), p(ws_conf),
                ws_conf.numel())))
        self.step_calls.append((lib.focus_select_queries, (
            p(self.conf), p(self.masked), n_gen, k_focus, window, 0, n_gen, p(self.focus_idx), p(self.active_idx), self.max_active,
            p(self.counts))))
        for l in range(n_layers):
            s = shape(self.q[l], self.k_cache[l], self.v_cache[l], self.out[l])
            self.step_calls.append((lib.focus_cache_update, (
                p(self.k_cache[l]), p(self.v_cache[l]), C.byref(s), p(self.k_new[l]), p(self.v_new[l]), self.k_new[l].stride(0),
                self.k_new[l].stride(1), p(self.active_idx), p(self.counts), self.max_active, row_base)))
            if l == l_dense:
                ws = workspace(fb.workspace_bytes(fb.FN_PROBE_LAYER, s, self.max_active))
                self.step_calls.append((lib.focus_probe_layer, (
                    p(self.q[l]), p(self.active_idx), p(self.counts), self.max_active, p(self.k_cache[l]), p(self.v_cache[l]),
                    C.byref(s), n_sink, p(self.out[l]), None, p(self.col_mass), p(self.sink_idx), p(ws), ws.numel())))
            elif self.is_sparse(l):
                ws = workspace(fb.workspace_bytes(fb.FN_SPARSE_LAYER, s, self.max_active, n_keep, n_sink))
                self.step_calls.append((lib.focus_sparse_layer, (
                    p(self.q[l]), p(self.focus_idx), p(self.active_idx), p(self.counts), k_focus, self.max_active,
                    p(self.k_cache[l]), p(self.v_cache[l]), p(self.kbar[l]), C.byref(s), n_keep, p(self.sink_idx), n_sink,
                    p(self.scores[l]), p(self.kept[l]), p(self.out[l]), None, p(ws), ws.numel())))
            else:
                ws = workspace(fb.workspace_bytes(fb.FN_SPARSE_ATTN, s, self.max_active, self.n_b, 0))
                self.step_calls.append((lib.focus_sparse_attn, (
                    p(self.q[l]), p(self.active_idx), p(self.counts), self.max_active, p(self.k_cache[l]), p(self.v_cache[l]),
                    C.byref(s), p(self.all_blocks), self.n_b, None, 0, p(self.out[l]), None, p(ws), ws.numel())))
        self._g_entry = self._g_step = None

    def is_sparse(self, l: int) -> bool:
        return self.l_dense < l < self.first_tail

    def run_entry(self):
        if self._g_entry is not None:
            self._g_entry.replay()
        else:
            FocusStep._issue(self.entry_calls, torch.cuda.current_stream().cuda_stream)

    def run_step(self):
        if self._g_step is not None:
            self._g_step.replay()
        else:
            FocusStep._issue(self.step_calls, torch.cuda.current_stream().cuda_stream)

    def capture(self):
        """Capture the block entry and the step into one HIP graph each (after one eager run of both, so that no module
        is loaded under capture).  The eager run executes a step on whatever the input buffers hold: call this before
        the first real block entry, or re-run the entry afterwards."""
        self._g_entry = self._g_step = None
        self.run_entry()
        self.run_step()
        torch.cuda.synchronize()
        graphs = []
        for calls in (self.entry_calls, self.step_calls):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                FocusStep._issue(calls, torch.cuda.current_stream().cuda_stream)
            graphs.append(g)
        self._g_entry, self._g_step = graphs
