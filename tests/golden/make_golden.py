"""Writes tests/golden/*.json: oracle results on the seeded workloads, stored as text.

The paper prints no numeric example of this path, so these files hold no paper values: they freeze what
the oracle (and only the oracle) computes on the committed seeds, so that a later change to the oracle's
arithmetic or to the input generator cannot pass unnoticed.  Run from the repo root:
    python tests/golden/make_golden.py
It imports nothing but the oracle and the input generator.
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import focus_inputs as fi  # noqa: E402
from oracle import focus_oracle as fo  # noqa: E402


def record(w):
    q, k, v = fi.layer_qkv(w, 0)
    Q, K, V = (x.float().numpy() for x in (q, k, v))
    conf = fi.confidence(w).numpy()
    focus = fo.select_focus(conf, None, w.k_focus)
    active = fo.expand_window(focus, w.window, 0, w.n_gen)
    S = fo.sink_scores(Q, active, K)
    sinks = fo.select_sinks(S, w.n_ctx, w.n_sink)
    lay = fo.focus_layer(Q, K, V, focus, active, sinks, w.n_ctx, w.block, w.n_keep)
    return {
        "workload": w.name, "seed": w.seed,
        "input_checksum": {n: int(fi.bf16_bits(t).astype(np.uint64).sum()) for n, t in (("q", q), ("k", k), ("v", v))},
        "focus": focus.tolist(), "active": active.tolist(), "sinks": sinks.tolist(), "blocks": lay["blocks"].tolist(),
        "margin_focus": fo.decision_margin(conf, w.k_focus),
        "margin_sinks": fo.decision_margin(S, w.n_sink, np.arange(len(S)) < w.n_ctx),
        "margin_blocks": fo.decision_margin(lay["R"], w.n_keep),
        "R_head": [float(x) for x in lay["R"][:8]],
        "S_at_sinks": [float(S[j]) for j in sinks],
        "out_h0_row0_head": [float(x) for x in lay["out"][0, 0, :8]],
        "out_abs_mean": float(np.abs(lay["out"]).mean()),
    }


if __name__ == "__main__":
    here = os.path.dirname(os.path.abspath(__file__))
    for w in (fi.TINY, fi.CTX8K):
        with open(os.path.join(here, w.name + ".json"), "w") as f:
            json.dump(record(w), f, indent=1)
            f.write("\n")
        print("wrote", w.name)
