"""The seeded input generator and the oracle on the committed workloads (CPU only)."""
import importlib.util
import json
import os

import numpy as np
import pytest
import torch

import focus_inputs as fi
from focus_inputs import rng
from oracle import focus_oracle as fo

HERE = os.path.dirname(os.path.abspath(__file__))


def test_streams_are_counter_based_and_reproducible():
    key = rng.stream_key(7, 1, 2)
    whole = rng.normal(key, 0, 1000)
    parts = torch.cat([rng.normal(key, 0, 400), rng.normal(key, 400, 600)])
    assert torch.equal(whole, parts)
    assert not torch.equal(whole, rng.normal(rng.stream_key(7, 1, 3), 0, 1000))
    u = rng.uniform(key, 0, 100000)
    assert 0.0 <= float(u.min()) and float(u.max()) < 1.0
    assert abs(float(u.mean()) - 0.5) < 5e-3 and abs(float(u.var()) - 1 / 12) < 2e-3
    assert abs(float(whole.mean())) < 0.1 and abs(float(whole.std()) - 1) < 0.06


def test_workload_table_matches_the_stated_configurations():
    assert (fi.TINY.n_heads, fi.TINY.head_dim, fi.TINY.n_ctx, fi.TINY.n_gen, fi.TINY.k_focus, fi.TINY.block,
            fi.TINY.n_keep, fi.TINY.n_sink) == (4, 64, 1024, 32, 8, 64, 4, 2)
    for w, m, c in ((fi.CTX8K, 8192, 6), (fi.CTX16K, 16384, 6), (fi.CTX32K, 32768, 7), (fi.STACK32K, 32768, 7)):
        assert (w.n_heads, w.head_dim, w.n_ctx, w.n_gen, w.n_resp, w.k_focus, w.block, w.n_keep, w.n_sink) == \
               (32, 128, m, 64, 64, 16, 128, c, 4)
        assert len(set(w.sink_positions)) == 4 and all(0 <= s < m for s in w.sink_positions)
    assert (fi.STACK32K.n_layers, fi.STACK32K.probe_layer, fi.STACK32K.first_sparse_layer) == (32, 16, 17)


def test_layer_tensors_shape_bias_and_determinism():
    w = fi.TINY
    q, k, v = fi.layer_qkv(w, 0)
    assert q.shape == (4, 32, 64) and k.shape == v.shape == (4, 1056, 64) and q.dtype == torch.bfloat16
    q2, k2, v2 = fi.layer_qkv(w, 0)
    assert torch.equal(q, q2) and torch.equal(k, k2) and torch.equal(v, v2)
    assert torch.equal(fi.layer_qkv(w, 0, which="k"), k)
    assert not torch.equal(fi.layer_qkv(w, 1, which="k"), k)
    u = fi.shared_direction(w)
    assert float(torch.linalg.vector_norm(u)) == pytest.approx(1.0, abs=1e-6)
    kf = k.float()
    proj = kf @ u                                   # [H, L]: N(0,1) everywhere except +4 at the planted rows
    assert float(proj[:, list(w.sink_positions)].mean()) == pytest.approx(4.0, abs=1.0)
    assert abs(float(proj[:, 2:].mean())) < 0.1
    assert float((q.float() @ u).mean()) == pytest.approx(0.5, abs=0.25)
    conf = fi.confidence(fi.CTX8K)
    assert conf.dtype == torch.float32 and conf.shape == (64,) and 0 <= float(conf.min()) and float(conf.max()) < 1


@pytest.mark.parametrize("name", ["tiny", "ctx8k"])
def test_oracle_reproduces_golden_file(name):
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    got = mod.record(fi.WORKLOADS[name])
    with open(os.path.join(HERE, "golden", name + ".json")) as f:
        ref = json.load(f)
    for key in ("input_checksum", "focus", "active", "sinks", "blocks"):
        assert got[key] == ref[key], key
    for key in ("R_head", "S_at_sinks", "out_h0_row0_head", "out_abs_mean"):
        assert np.allclose(got[key], ref[key], rtol=1e-9, atol=1e-12), key
    # index parity against a fp32 GPU path is only well posed when no decision is a near-tie
    for key in ("margin_focus", "margin_sinks", "margin_blocks"):
        assert got[key] > 1e-4, (key, got[key])


def test_strong_sink_variant_makes_planted_keys_the_sinks():
    w = fi.strong_sinks(fi.TINY)
    q, k, _ = fi.layer_qkv(w, 0)
    Q, K = q.float().numpy(), k.float().numpy()
    active = fo.select_focus(fi.confidence(w).numpy(), None, w.k_focus)
    S = fo.sink_scores(Q, active, K)
    assert fo.select_sinks(S, w.n_ctx, w.n_sink).tolist() == list(w.sink_positions)
    assert S[list(w.sink_positions)].sum() > 0.2      # they hold a large share of all attention mass
