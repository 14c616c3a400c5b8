#!/usr/bin/env python3
"""Benchmark of the Focus-dLLM sparse-attention step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload stack32k]

A "step" is one pass of the whole hot path over the 32-layer, 32K-context workload: query selection once,
sink identification once at the probe layer (16), then for each of the 15 sparse layers (17..31) one
focus_sparse_layer call (K scan -> block relevance, Top-C, sparse attention).  All inputs are resident in HBM
before the clock starts.  Prints ONE JSON line: `value` = ms per step with nothing cached between steps; the same
step with cached block means and with dense attention; per-stage microseconds, GB/s and TFLOP/s against the
algorithmic bytes and flops; `roofline` for the stage with the largest share of the step; `roofline_block_entry`: one
layer of a block entry (dense attention of every position, not part of the step) against the bf16 MFMA peak;
`cpu_baseline`: the float64 oracle timed on the host; `parity_vs_oracle`: a spot check of the timed buffers.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0


PMC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_{}.json")


def parse_pmc(fetch_db: str, write_db: str, workload: str) -> int:
    """Per-kernel HBM traffic from two `rocprofv3 --pmc` runs of `bench.py --mode pmc` (FETCH_SIZE, then WRITE_SIZE;
    both in KiB per dispatch), each scaled by what the same counter reads for the 1 GiB calibration copy."""
    import sqlite3

    def per_kernel(db, counter):
        c = sqlite3.connect(db)
        rows = c.execute("select kernel_name, counter_name, value from counters_collection").fetchall() \
            if any(r[0] == "counters_collection" for r in c.execute("select name from sqlite_master")) else []
        out = {}
        for name, cname, value in rows:
            if cname != counter:
                continue
            out.setdefault(name, []).append(float(value))
        return out

    fetch, write = per_kernel(fetch_db, "FETCH_SIZE"), per_kernel(write_db, "WRITE_SIZE")
    copy_bytes = float(1 << 30)

    def copy_kernel(d):
        cands = [(max(v), k) for k, v in d.items() if "elementwise" in k or "copy" in k.lower()]
        return max(cands)[1] if cands else None

    kf, kw = copy_kernel(fetch), copy_kernel(write)
    f_scale = copy_bytes / (max(fetch[kf]) * 1024.0) if kf else 1.0   # true bytes per counted byte
    w_scale = copy_bytes / (max(write[kw]) * 1024.0) if kw else 1.0
    res = {"workload": workload, "unit": "bytes per dispatch", "calibration": {
        "copy_bytes": copy_bytes, "copy_kernel_fetch": kf, "copy_kernel_write": kw,
        "FETCH_SIZE_KiB_for_copy": max(fetch[kf]) if kf else None, "WRITE_SIZE_KiB_for_copy": max(write[kw]) if kw else None,
        "fetch_scale": f_scale, "write_scale": w_scale}, "kernels": {}}
    for name in sorted(set(fetch) | set(write)):
        if "focus::" not in name:
            continue
        f = fetch.get(name, [0.0])
        wv = write.get(name, [0.0])
        # the largest dispatch of a kernel name is the full-size one (dense attention shares a name with sparse)
        res["kernels"][name] = {"dispatches": len(f), "fetch_bytes_max": max(f) * 1024 * f_scale, "fetch_bytes_min": min(f) * 1024 * f_scale,
                                "write_bytes_max": max(wv) * 1024 * w_scale, "write_bytes_min": min(wv) * 1024 * w_scale}
    path = PMC_FILE.format(workload)
    with open(path, "w") as fh:
        json.dump(res, fh, indent=1)
        fh.write("\n")
    print("wrote", path)
    return 0


def parse_mfma(db: str, workload: str) -> int:
    """MFMA utilisation per kernel from one `rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_INSTS_VALU_MFMA_MOPS_BF16
    SQ_BUSY_CYCLES GRBM_GUI_ACTIVE` run of `bench.py --mode pmc`.  Prints a markdown table:
    util = MFMA-busy cycles / (GPU-active cycles x 4 SIMDs x 256 CUs); flops = MOPS x 512; the last column prices the
    same flops against the dense bf16 peak over the GPU-active time at 2.4 GHz."""
    import sqlite3
    c = sqlite3.connect(db)
    cols = [d[0] for d in c.execute("select * from counters_collection limit 1").description]
    disp = "dispatch_id" if "dispatch_id" in cols else ("correlation_id" if "correlation_id" in cols else None)
    if disp is None:
        print("no dispatch column in counters_collection; columns:", cols)
        return 1
    # rocprofv3 returns one value per (dispatch, counter), already summed over the hardware instances: event counts
    # are then totals, while the cycle counter GRBM_GUI_ACTIVE is the sum over the chip's 8 XCDs (its reading for a
    # kernel of known duration confirms this: 8 x duration x clock) and is divided by 8 to get GPU-active cycles
    rows = c.execute(f"select {disp}, kernel_name, counter_name, sum(value) from counters_collection "
                     f"group by {disp}, kernel_name, counter_name").fetchall()
    per = {}
    for d, name, cname, v in rows:
        if "focus::" in name:
            per.setdefault((name, d), {})[cname] = float(v) / (8.0 if cname == "GRBM_GUI_ACTIVE" else 1.0)
    by_kernel = {}
    for (name, d), cs in per.items():
        by_kernel.setdefault(name, []).append(cs)
    print(f"workload {workload}; one row per kernel: mean over its dispatches, and the largest dispatch (by MFMA work)\n")
    print("| kernel | dispatches | MFMA busy cycles (sum over SIMDs) | GPU active cycles | MFMA util % | bf16 MFMA flops | largest dispatch: util % / flops | flops / (active time x 2.5 PFLOP/s) % |")
    print("|---|---|---|---|---|---|---|---|")
    n_simd = 256 * 4
    for name in sorted(by_kernel):
        ds = by_kernel[name]
        g = lambda cs, k: cs.get(k, 0.0)
        util = lambda cs: 100.0 * g(cs, "SQ_VALU_MFMA_BUSY_CYCLES") / max(g(cs, "GRBM_GUI_ACTIVE") * n_simd, 1.0)
        mean = lambda k: sum(g(cs, k) for cs in ds) / len(ds)
        big = max(ds, key=lambda cs: g(cs, "SQ_INSTS_VALU_MFMA_MOPS_BF16"))
        short = name.replace("void focus::", "").replace("focus::", "").split("(")[0]
        print(f"| `{short}` | {len(ds)} | {mean('SQ_VALU_MFMA_BUSY_CYCLES'):.0f} | {mean('GRBM_GUI_ACTIVE'):.0f} | "
              f"{sum(util(cs) for cs in ds) / len(ds):.2f} | {mean('SQ_INSTS_VALU_MFMA_MOPS_BF16') * 512:.3e} | "
              f"{util(big):.2f} / {g(big, 'SQ_INSTS_VALU_MFMA_MOPS_BF16') * 512:.3e} | "
              f"{100.0 * mean('SQ_INSTS_VALU_MFMA_MOPS_BF16') * 512 / max(mean('GRBM_GUI_ACTIVE') / 2.4e9 * MFMA_BF16_PEAK_TFLOPS * 1e12, 1.0):.2f} |")
    return 0


def parse_trace(db: str) -> int:
    """Per-kernel duration table from a `rocprofv3 --kernel-trace --stats` result database of a bench.py run.
    Launches are grouped by (kernel, grid) because the dense comparison runs through the same kernel as the sparse path."""
    import sqlite3
    c = sqlite3.connect(db)
    rows = c.execute("select name, grid_x, grid_y, grid_z, count(*), avg(end-start), min(end-start), max(end-start), sum(end-start) "
                     "from kernels where name like '%focus::%' group by name, grid_x, grid_y, grid_z order by sum(end-start) desc").fetchall()
    print(f"| kernel | grid (threads) | launches | avg us | min us | max us | total ms |")
    print("|---|---|---|---|---|---|---|")
    for n, gx, gy, gz, cnt, avg, mn, mx, sm in rows:
        short = n.replace("void focus::", "").replace("focus::", "").split("(")[0]
        print(f"| `{short}` | {gx}x{gy}x{gz} | {cnt} | {avg / 1e3:.2f} | {mn / 1e3:.2f} | {mx / 1e3:.2f} | {sm / 1e6:.3f} |")
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="stack32k", choices=["stack32k", "ctx32k", "ctx16k", "ctx8k", "tiny", "paper32k", "paper32k_gen256", "ctx128k"])
    ap.add_argument("--sets", type=int, default=2, help="independent copies of the layer tensors rotated between steps "
                    "so that no step finds its K/V in the 256 MB Infinity Cache")
    ap.add_argument("--no-graph", action="store_true", help="enqueue every call eagerly instead of replaying a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--kernel-reps", type=int, default=4)
    ap.add_argument("--full-refresh", action="store_true", help="kept for old command lines: the block-entry layer is timed by default")
    ap.add_argument("--no-full-refresh", action="store_true",
                    help="skip timing one layer of a block-entry refresh (dense attention of all M+N positions, the MFMA-bound case)")
    ap.add_argument("--mode", default="bench", choices=["bench", "pmc"],
                    help="pmc: run a 1 GiB copy (calibration) and a few launches of every stage, nothing else; meant to be "
                         "run under `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE`")
    ap.add_argument("--parse-pmc", nargs=2, metavar=("FETCH_DB", "WRITE_DB"),
                    help="turn the two rocprofv3 --pmc result databases of a `--mode pmc` run into profiles/hbm_traffic_<workload>.json")
    ap.add_argument("--parse-mfma", metavar="DB", help="print the MFMA utilisation table of a rocprofv3 --pmc database (see parse_mfma)")
    ap.add_argument("--parse-trace", metavar="DB", help="print the per-kernel table of a rocprofv3 --kernel-trace database")
    args = ap.parse_args()
    if args.parse_trace:
        return parse_trace(args.parse_trace)
    if args.parse_mfma:
        return parse_mfma(args.parse_mfma, args.workload)
    if args.parse_pmc:
        return parse_pmc(args.parse_pmc[0], args.parse_pmc[1], args.workload)
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path has no multi-GPU part); run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import focus_inputs as fi
    from paper_2602_02159_amd import binding as fb
    from paper_2602_02159_amd.step import FocusStep

    fb.lib()  # fail loudly when the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = fi.WORKLOADS[args.workload]
    if w.n_layers == 1:
        probe_layer, sparse_ids = 0, [0]
    else:
        probe_layer, sparse_ids = w.probe_layer, list(range(w.first_sparse_layer, w.n_layers))
    n_sparse = len(sparse_ids)

    # ---- inputs, generated on the device from the seeded counter-based streams; `sets` independent copies
    t0 = time.time()
    conf = fi.confidence(w, dev)
    masked = fi.masked_all(w, dev)
    steps_obj = []
    for s in range(args.sets):
        ws_ = w.with_(seed=w.seed + 7919 * s)
        probe = fi.layer_qkv(ws_, probe_layer, dev, which="qkv")
        layers = [fi.layer_qkv(ws_, l, dev) for l in sparse_ids]
        steps_obj.append(FocusStep(conf, masked, probe, layers, w.n_ctx, w.block, w.k_focus, w.window, w.n_keep, w.n_sink))
    torch.cuda.synchronize()
    gen_s = time.time() - t0

    def sync():
        torch.cuda.synchronize()

    if args.mode == "pmc":
        # calibration: a plain device-to-device copy of known size, then every stage a few times on distinct layers
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)   # an elementwise kernel that reads 1 GiB and writes 1 GiB
        sync()
        st = steps_obj[0]
        st.run()
        sync()
        for stage in ("block_means", "block_partials", "block_scores_cached", "sparse_attn", "dense_attn", "find_sinks", "probe_layer",
                      "select"):
            st.issue(stage)
            sync()
        # block entry: the cache rewrite, and the dense attention of every position at an eighth of the query rows
        # (the counters are ratios; a launch over all rows would run twenty times longer under the profiler)
        q0, k0, v0 = st.layers[0]
        kc, vc = torch.empty_like(k0), torch.empty_like(v0)
        kb = torch.empty(w.n_heads, w.n_blocks, w.head_dim, dtype=torch.float32, device=dev)
        fb.cache_refresh(kc, vc, fb.make_shape(q0, kc, vc, w.n_ctx, w.block), k0, v0, kb)
        sync()
        q_part = torch.randn(w.n_heads, w.n_kv // 8, w.head_dim, device=dev).to(torch.bfloat16)
        o_part = torch.empty_like(q_part)
        fb.refresh_attn(q_part, k0, v0, fb.make_shape(q_part, k0, v0, w.n_ctx, w.block, o_part), o_part, None)
        sync()
        print(json.dumps({"mode": "pmc", "copy_bytes": int(src.numel() * 4), "workload": w.name}))
        return 0

    # ---- eager run once: results used for the parity spot check and the byte counts
    for st in steps_obj:
        st.run()
    sync()
    st0 = steps_obj[0]
    sinks = st0.sink_idx.cpu().tolist()
    kept = [b["kept"].cpu().tolist() for b in st0.bufs]
    n_keys = []
    for kb in kept:
        rows = set(j for j in sinks if 0 <= j < w.n_ctx)
        for b in kb:
            rows.update(range(b * w.block, min((b + 1) * w.block, w.n_ctx)))
        n_keys.append(len(rows) + w.n_resp)
    n_q = int(st0.counts.cpu()[1])
    H, d, L, M = w.n_heads, w.head_dim, w.n_kv, w.n_ctx
    n_b = w.n_blocks

    # ---- algorithmic bytes / flops per launch of each stage: what the method must move, not what an implementation
    # may add (the logits spilled, or K read a second time, while scoring the sinks are not counted)
    mean_keys = float(np.mean(n_keys))
    alg = {
        "select": {"bytes": w.n_gen * 5 + 4 * (w.k_focus + n_q + 2), "flops": 0},
        "find_sinks": {"bytes": L * H * d * 2 + n_q * H * d * 2 + L * 4, "flops": 2 * n_q * L * d * H},
        "block_means": {"bytes": M * H * d * 2 + n_b * H * d * 4, "flops": M * H * d},
        "block_partials": {"bytes": M * H * d * 2 + w.k_focus * H * d * 2 + n_b * H * 4, "flops": M * H * d + 2 * n_b * d * H},
        "block_scores_cached": {"bytes": n_b * H * d * 4 + w.k_focus * H * d * 2 + n_b * 4, "flops": 2 * n_b * d * H},
        "sparse_attn": {"bytes": 2 * mean_keys * H * d * 2 + 2 * n_q * H * d * 2, "flops": 4 * n_q * mean_keys * d * H},
        "dense_attn": {"bytes": 2 * L * H * d * 2 + 2 * n_q * H * d * 2, "flops": 4 * n_q * L * d * H},
        # the probe layer's own dense attention with the sinks as a by-product: K and V once
        "probe_layer": {"bytes": 2 * L * H * d * 2 + 2 * n_q * H * d * 2 + L * 4, "flops": 4 * n_q * L * d * H},
    }
    # scoring from raw K: the scan emits the per-head partial relevances directly (no means are stored), then Top-C
    alg["block_scores"] = {"bytes": alg["block_partials"]["bytes"] + n_b * H * 4 + n_b * 4, "flops": alg["block_partials"]["flops"]}
    alg["sparse_layer_cached"] = {"bytes": alg["block_scores_cached"]["bytes"] + alg["sparse_attn"]["bytes"],
                                  "flops": alg["block_scores_cached"]["flops"] + alg["sparse_attn"]["flops"]}
    alg["sparse_layer"] = {"bytes": alg["block_scores"]["bytes"] + alg["sparse_attn"]["bytes"],
                           "flops": alg["block_scores"]["flops"] + alg["sparse_attn"]["flops"]}

    # ---- HIP graph of the step (validated against the eager results over several replays)
    use_graph = not args.no_graph
    if use_graph:
        try:
            ref_out = [b["out"].clone() for b in st0.bufs]
            ref_kept = [b["kept"].clone() for b in st0.bufs]
            for st in steps_obj:
                st.capture()
            for rep in range(3):
                for b in st0.bufs:
                    b["out"].zero_()
                    b["kept"].fill_(-5)
                sync()
                st0.run()
                sync()
                ok = all(torch.equal(a, b["out"]) for a, b in zip(ref_out, st0.bufs)) and \
                    all(torch.equal(a, b["kept"]) for a, b in zip(ref_kept, st0.bufs))
                if not ok:
                    raise RuntimeError(f"graph replay {rep} differs from the eager result")
        except Exception as e:  # fall back to eager launches, and say so in the output
            print(f"bench.py: HIP graph disabled ({e})", file=sys.stderr)
            for st in steps_obj:
                st.release_graph()
            use_graph = False

    def time_steps(objs, n, warm):
        for i in range(warm):
            objs[i % len(objs)].run()
        sync()
        t = time.perf_counter()
        for i in range(n):
            objs[i % len(objs)].run()
        sync()
        return (time.perf_counter() - t) * 1e3 / n

    # ---- the timed region: exactly K steps, every stage recomputed every step (nothing cached between steps)
    ms_step = time_steps(steps_obj, args.steps, args.warmup)

    # ---- secondary timings (same run): block means cached across steps; the same layers with dense attention
    def variant(cached_means=False, dense=False):
        objs = []
        for st in steps_obj:
            v = FocusStep.__new__(FocusStep)
            v.__dict__.update(st.__dict__)
            v.cached_means, v.dense, v._graph = cached_means, dense, None
            if use_graph:
                v.capture()
            objs.append(v)
        return objs

    for st in steps_obj:
        st.issue("block_means")
    sync()
    ms_cached = time_steps(variant(cached_means=True), args.steps, args.warmup)
    ms_dense = time_steps(variant(dense=True), max(5, args.steps // 5), 2)

    # ---- per-stage durations with HIP events on the launch stream, back to back over all layers of all sets
    def time_stage(stage):
        n_launch = 0
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for st in steps_obj:
            st.issue(stage)
        sync()
        e0.record()
        for _ in range(args.kernel_reps):
            for st in steps_obj:
                st.issue(stage)
                n_launch += len(st.calls[stage])
        e1.record()
        sync()
        return e0.elapsed_time(e1) * 1e3 / n_launch  # microseconds per launch

    stages = {}
    per_step_count = {"select": 1, "find_sinks": 1, "block_means": n_sparse, "block_partials": n_sparse, "block_scores_cached": n_sparse,
                      "block_scores": n_sparse, "sparse_attn": n_sparse, "dense_attn": n_sparse, "sparse_layer": n_sparse,
                      "sparse_layer_cached": n_sparse, "probe_layer": 0}
    for stage in ("select", "find_sinks", "block_means", "block_partials", "block_scores_cached", "block_scores", "sparse_attn", "dense_attn",
                  "sparse_layer_cached", "sparse_layer", "probe_layer"):
        us = time_stage(stage)
        a = alg[stage]
        stages[stage] = {"us_per_launch": round(us, 3), "launches_per_step": per_step_count[stage],
                         "alg_bytes": int(a["bytes"]), "alg_flops": int(a["flops"]),
                         "GBps": round(a["bytes"] / us * 1e-3, 1), "TFLOPps": round(a["flops"] / us * 1e-6, 3),
                         "hbm_frac": round(a["bytes"] / us * 1e-3 / HBM_PEAK_GBS, 4)}

    # ---- the two operations around the step (not part of `value`): confidence from vocabulary logits (Eq. 2) for the
    # generation block, and the KV-cache refresh of the active rows (Eq. 3) of one layer
    def time_call(fn, reps=32, replays=5):   # a graph of `reps` calls: the host's per-call cost stays out of the figure
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        fn()
        sync()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(reps):
                fn()
        g.replay()
        sync()
        e0.record()
        for _ in range(replays):
            g.replay()
        e1.record()
        sync()
        return e0.elapsed_time(e1) * 1e3 / (reps * replays)

    vocab = 126464
    vl = [torch.randn(w.n_gen, vocab, device=dev).mul_(3.0).to(torch.bfloat16) for _ in range(4)]   # 4 x 16 MB, rotated
    tok_buf = torch.empty(w.n_gen, dtype=torch.int32, device=dev)
    conf_buf = torch.empty(w.n_gen, dtype=torch.float32, device=dev)
    conf_ws = torch.empty(max(fb.token_confidence_workspace(w.n_gen, vocab), 16), dtype=torch.uint8, device=dev)
    rot = [0]

    def conf_call():
        rot[0] = (rot[0] + 1) % len(vl)
        fb.token_confidence(vl[rot[0]], masked, tok_buf, conf_buf, conf_ws)
    us = time_call(conf_call)
    cb = w.n_gen * vocab * 2
    stages["token_confidence"] = {"us_per_launch": round(us, 3), "launches_per_step": 0, "alg_bytes": cb, "alg_flops": 0,
                                  "GBps": round(cb / us * 1e-3, 1), "TFLOPps": 0.0, "hbm_frac": round(cb / us * 1e-3 / HBM_PEAK_GBS, 4),
                                  "shape": f"{w.n_gen} x {vocab} bf16 logits"}
    q0, k0, v0 = st0.layers[0]
    k_new = torch.randn(H, st0.max_active, d, device=dev).to(torch.bfloat16)
    v_new = torch.randn(H, st0.max_active, d, device=dev).to(torch.bfloat16)
    k_cache, v_cache = k0.clone(), v0.clone()
    s_cache = fb.make_shape(q0, k_cache, v_cache, M, w.block)
    us = time_call(lambda: fb.cache_update(k_cache, v_cache, s_cache, k_new, v_new, st0.active_idx, st0.counts, M))
    ub = 2 * 2 * n_q * H * d * 2
    stages["cache_update"] = {"us_per_launch": round(us, 3), "launches_per_step": 0, "alg_bytes": ub, "alg_flops": 0,
                              "GBps": round(ub / us * 1e-3, 1), "TFLOPps": 0.0, "hbm_frac": round(ub / us * 1e-3 / HBM_PEAK_GBS, 4)}
    # block entry: every cache row rewritten, block means from the same pass (reads K, V; writes K, V, K_bar)
    kbar_r = torch.empty(H, n_b, d, dtype=torch.float32, device=dev)
    us = time_call(lambda: fb.cache_refresh(k_cache, v_cache, s_cache, k0, v0, kbar_r))
    ub = 2 * 2 * L * H * d * 2 + H * n_b * d * 4
    stages["cache_refresh"] = {"us_per_launch": round(us, 3), "launches_per_step": 0, "alg_bytes": ub, "alg_flops": 0,
                               "GBps": round(ub / us * 1e-3, 1), "TFLOPps": 0.0, "hbm_frac": round(ub / us * 1e-3 / HBM_PEAK_GBS, 4)}
    del vl, k_cache, v_cache, kbar_r
    if not args.no_full_refresh:
        # block entry (Alg. 1): every position is active and attends to every key; 4 L^2 d H flops against the bf16 MFMA peak
        q_all = torch.randn(H, L, d, device=dev).to(torch.bfloat16)
        out_all = torch.empty(H, L, d, dtype=torch.bfloat16, device=dev)
        s_all = fb.make_shape(q_all, k0, v0, M, w.block, out_all)
        call = lambda: fb.refresh_attn(q_all, k0, v0, s_all, out_all, None)
        call()
        sync()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(3):
            call()
        e1.record()
        sync()
        us = e0.elapsed_time(e1) * 1e3 / 3
        fl = 4 * L * L * d * H
        stages["full_refresh_layer"] = {"us_per_launch": round(us, 1), "launches_per_step": 0, "alg_bytes": int(2 * 2 * L * H * d * 2),
                                        "alg_flops": int(fl), "GBps": round(2 * 2 * L * H * d * 2 / us * 1e-3, 1),
                                        "TFLOPps": round(fl / us * 1e-6, 1), "mfma_frac": round(fl / us * 1e-6 / MFMA_BF16_PEAK_TFLOPS, 4),
                                        "bound": "mfma"}
        del q_all, out_all

    # the stage that takes the largest share of the timed step
    # (the step calls focus_sparse_layer; its parts are also timed through the separate entry points, which run the same kernels)
    in_step = ("select", "find_sinks", "block_partials", "sparse_attn")
    share = {s: stages[s]["us_per_launch"] * per_step_count[s] for s in in_step}
    dom_kernel = max(share, key=share.get)
    ds = stages[dom_kernel]
    cap_q = st0.max_active                              # the launchers plan for the capacity of the active list
    qtw = 1 if cap_q <= 16 else (2 if cap_q <= 32 else 4)   # query tiles per workgroup they pick
    kernel_name = {"block_partials": f"block_means_kernel<{d}, true>",
                   "find_sinks": f"qk_logits_kernel<{d}, {qtw}, {0 if qtw == 1 else 1}> and the rest of the sink chain",
                   "sparse_attn": f"sparse_attn_kernel<{d}, {qtw}, 1>", "select": "select_queries_kernel"}[dom_kernel]
    # HBM traffic of that kernel, measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE in a separate run of this
    # script (--mode pmc) and stored by --parse-pmc; scaled by the counters' reading for a 1 GiB copy
    traffic = None
    try:
        with open(PMC_FILE.format(w.name)) as fh:
            pmc = json.load(fh)
        # the counters are taken on the stand-alone stages; the attention kernel appears there without the fused Top-C
        # prologue (<128, 1, 0>), a name the dense comparison shares: its smallest dispatch is the sparse one
        want = [f"sparse_attn_kernel<{d}, {qtw}, 0>" if dom_kernel == "sparse_attn" else kernel_name.split(" and ")[0]]
        if dom_kernel == "find_sinks":   # every kernel of the chain: logits (one or two passes over K), row statistics, column mass, Top-N
            want += ["lse_combine_kernel", "column_mass_kernel", "sink_final_kernel", "sink_select_kernel", "reduce_topk_kernel<0>"]
            if qtw > 1:
                want.append(f"qk_logits_kernel<{d}, {qtw}, 2>")
        which = "min" if dom_kernel == "sparse_attn" else "max"
        for name, v in pmc["kernels"].items():
            if any(x in name for x in want):
                traffic = (traffic or 0) + int(v[f"fetch_bytes_{which}"] + v[f"write_bytes_{which}"])
    except (OSError, KeyError, ValueError):
        pass
    roofline = {"bound": "hbm", "kernel": kernel_name, "achieved": ds["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": ds["hbm_frac"], "traffic": traffic, "us_per_launch": ds["us_per_launch"],
                "alg_bytes_per_launch": ds["alg_bytes"]}

    step_bytes = alg["select"]["bytes"] + alg["find_sinks"]["bytes"] + n_sparse * (alg["block_scores"]["bytes"] + alg["sparse_attn"]["bytes"])
    step_flops = alg["find_sinks"]["flops"] + n_sparse * (alg["block_scores"]["flops"] + alg["sparse_attn"]["flops"])
    cached_bytes = alg["select"]["bytes"] + alg["find_sinks"]["bytes"] + n_sparse * alg["sparse_layer_cached"]["bytes"]

    # ---- parity spot check + CPU baseline: the oracle on the probe layer and the first sparse layers of set 0
    cpu = None
    parity = None
    if not args.no_cpu_baseline:
        from oracle import focus_oracle as fo
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        to_np = lambda t: t.float().cpu().numpy()
        n_sample = min(3, n_sparse)
        Qp, Kp = to_np(st0.probe[0]), to_np(st0.probe[1])
        sample = [tuple(to_np(t) for t in st0.layers[i]) for i in range(n_sample)]
        conf_np = conf.cpu().numpy()
        t = time.perf_counter()
        focus_ref = fo.select_focus(conf_np, None, w.k_focus)
        active_ref = fo.expand_window(focus_ref, w.window, 0, w.n_gen)
        sinks_ref = fo.select_sinks(fo.sink_scores(Qp, active_ref, Kp), w.n_ctx, w.n_sink)
        t_once = time.perf_counter() - t
        t = time.perf_counter()
        lays = [fo.focus_layer(Q, K, V, focus_ref, active_ref, sinks_ref, w.n_ctx, w.block, w.n_keep) for Q, K, V in sample]
        t_layer = (time.perf_counter() - t) / n_sample
        cpu_ms = (t_once + n_sparse * t_layer) * 1e3
        cpu = {"value": round(cpu_ms, 1), "unit": "ms", "cores": int(cores), "kind": "oracle",
               "sample": f"query selection + sink identification on the probe layer, and {n_sample} of the {n_sparse} sparse layers "
                         f"(block means, relevance, Top-C, attention), float64 numpy; layer time scaled to {n_sparse} layers"}
        st0.release_graph()
        st0.run()
        sync()
        err = [np.abs(to_np(st0.bufs[i]["out"])[:, :n_q] - lays[i]["out"]) for i in range(n_sample)]   # rows past |I_active| are padding
        parity = {
            "focus_idx": st0.focus_idx.cpu().tolist() == focus_ref.tolist(),
            "sink_idx": st0.sink_idx.cpu().tolist() == sinks_ref.tolist(),
            "kept_blocks": all(st0.bufs[i]["kept"].cpu().tolist() == lays[i]["blocks"].tolist() for i in range(n_sample)),
            "attn_max_abs_err": float(max(e.max() for e in err)), "attn_mean_abs_err": float(np.mean([e.mean() for e in err])),
        }

    out = {
        "metric": "sparse-attn step latency at 32K ctx" if "32k" in w.name else f"sparse-attn step latency ({w.name})",
        "value": round(ms_step, 4), "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "layers_in_step": f"probe {probe_layer} + sparse {sparse_ids[0]}..{sparse_ids[-1]}",
                   "heads": H, "head_dim": d, "n_ctx": M, "n_resp": w.n_resp, "block": w.block, "n_queries": n_q,
                   "n_keep": w.n_keep, "n_sink": w.n_sink, "mean_keys_attended": mean_keys, "launch": "hip_graph" if use_graph else "eager",
                   "input_sets_rotated": args.sets, "block_means": "recomputed every step",
                   "per_layer_call": "focus_sparse_layer (K scan -> partial relevances, attention with Top-C inside, combine: three launches)"},
        "achieved_hbm_GBps": round(step_bytes / ms_step * 1e-6, 1), "achieved_TFLOPps": round(step_flops / ms_step * 1e-9, 3),
        "step_hbm_frac": round(step_bytes / ms_step * 1e-6 / HBM_PEAK_GBS, 4),
        "ms_per_step_block_means_cached": round(ms_cached, 4),
        "cached_step_hbm_GBps": round(cached_bytes / ms_cached * 1e-6, 1),
        "ms_per_step_dense_attention": round(ms_dense, 4),
        "dense_over_sparse": round(ms_dense / ms_cached, 2),
        "paper_speedup_context": ">29x end-to-end decoding speedup over vanilla at 32K on NVIDIA H200 (whole 8B model; not comparable)",
        "roofline": roofline,
        # not part of the step: the one MFMA-bound launch of the method (block entry, every position attends to every key)
        "roofline_block_entry": None if "full_refresh_layer" not in stages else {
            "bound": "mfma", "kernel": f"refresh_attn_kernel<{d}, 1, 8>", "achieved": stages["full_refresh_layer"]["TFLOPps"],
            "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": stages["full_refresh_layer"]["mfma_frac"],
            "us_per_launch": stages["full_refresh_layer"]["us_per_launch"], "flops_per_launch": stages["full_refresh_layer"]["alg_flops"]},
        "stages": stages, "cpu_baseline": cpu, "parity_vs_oracle": parity, "input_gen_s": round(gen_s, 1),
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
