"""Sequencing of the C-ABI calls for one denoising step over a stack of layers (Alg. 1 of the paper).

Nothing is computed here: the class owns the device buffers (index sets, scores, outputs, workspaces),
marshals every call's arguments once, and `run` enqueues the library calls in the order the algorithm
prescribes, all on the current stream, with no host synchronisation between them — the index sets produced
by one call are consumed on the device by the next.  Because a step is a fixed sequence of launches on
fixed buffers it can also be captured into a HIP graph (`capture`) and replayed.
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
