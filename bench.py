#!/usr/bin/env python3
"""Benchmark of the Focus-dLLM sparse-attention step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload stack32k]

A "step" is one non-block-entry denoising step (Alg. 1) over the 32-layer, 32K-context workload: query selection
once, sink identification once at the probe layer (16), then for each of the 15 sparse layers (17..31) one
focus_sparse_layer call (block relevance from the block means cached at the block entry, Top-C, sparse attention).
Before the clock starts the block entry is played once: focus_cache_refresh writes every layer's K/V cache and emits
the block means K_bar, which stay frozen until the next block entry (Eq. 3: prompt keys are not refreshed in between).
All inputs are resident in HBM.  Prints ONE JSON line: `value` = ms per step; beside it the same step with the block
means recomputed from K in every layer and step, with dense attention, and with warm caches; per-stage microseconds,
GB/s and TFLOP/s against the algorithmic bytes and flops; `roofline` for the stage with the largest share of the step
(the sparse attention); `roofline_paper32k`: the sparse attention at the paper's own hyper-parameters;
`roofline_block_entry`: one layer of a block entry (dense attention of every position, not part of the step) against
the bf16 MFMA peak; `cpu_baseline`: the float64 oracle timed on the host; `parity_vs_oracle`: the timed buffers of
every layer against the oracle (a mismatch makes the script exit non-zero).
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


def parse_clock(db: str) -> int:
    """Shader clock during the long launches of `bench.py --mode refresh` from one `rocprofv3 --pmc GRBM_GUI_ACTIVE` run:
    the counter comes back summed over the 8 XCDs; cycles / 8 / duration is the clock the launch actually ran at."""
    import sqlite3
    c = sqlite3.connect(db)
    rows = c.execute("select dispatch_id, kernel_name, counter_name, sum(value), min(start), max(end) from counters_collection "
                     "where counter_name = 'GRBM_GUI_ACTIVE' group by dispatch_id, kernel_name order by dispatch_id").fetchall()
    print("| dispatch | kernel | duration ms | GPU-active cycles (per XCD) | clock GHz |")
    print("|---|---|---|---|---|")
    for d, name, _, v, t0, t1 in rows:
        dur = (t1 - t0) * 1e-9
        if dur < 2e-3:      # the long launches only: the attention of a whole layer and the 8192^3 products
            continue
        short = name.replace("void focus::", "").replace("focus::", "").split("(")[0][:60]
        print(f"| {d} | `{short}` | {dur * 1e3:.2f} | {v / 8:.3e} | {v / 8 / dur * 1e-9:.2f} |")
    return 0


def refresh_mode(args) -> int:
    """Block-entry attention of one 32K layer on normal-distributed and on all-zero inputs, next to the vendor library's
    plain bf16 product of 8192^3 on the same two kinds of input: the evidence for what bounds refresh_attn_kernel."""
    import torch

    import focus_inputs as fi
    from paper_2602_02159_amd import binding as fb
    dev = torch.device("cuda:0")
    w = fi.WORKLOADS["stack32k"]
    H, d, L, M = w.n_heads, w.head_dim, w.n_kv, w.n_ctx

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps   # ms

    res = {"mode": "refresh", "shape": f"H={H} L={L} d={d}"}
    fl = 4 * L * L * d * H
    for kind in ("normal", "zeros"):
        mk = (lambda *s: torch.randn(*s, device=dev).to(torch.bfloat16)) if kind == "normal" else \
             (lambda *s: torch.zeros(*s, dtype=torch.bfloat16, device=dev))
        q, k, v = mk(H, L, d), mk(H, L, d), mk(H, L, d)
        out = torch.empty_like(q)
        sh = fb.make_shape(q, k, v, M, w.block, out)
        ms = timed(lambda: fb.refresh_attn(q, k, v, sh, out, None), 3)
        res[f"refresh_attn_{kind}"] = {"ms": round(ms, 3), "TFLOPps": round(fl / ms * 1e-9, 1), "frac_of_2500": round(fl / ms * 1e-9 / 2500.0, 4)}
        del q, k, v, out
        a, b = mk(8192, 8192), mk(8192, 8192)
        ms = timed(lambda: torch.matmul(a, b), 10)
        res[f"matmul_8192_{kind}"] = {"ms": round(ms, 3), "TFLOPps": round(2 * 8192 ** 3 / ms * 1e-9, 1)}
        del a, b
    print(json.dumps(res))
    return 0


def decoder_mode(args) -> int:
    """Alg. 1 over a generation block of the whole 32-layer stack at the 32K shape, through FocusDecoder's two HIP graphs:
    the block entry (per layer: caches rewritten + block means, dense attention of every position) and one step (selection,
    then per layer the cache update of the active rows and dense attention up to the probe layer, the probe layer, the sparse
    layers from the block means of the entry).  Inputs: normal-distributed bf16 states, uniform confidences.  Not the
    driver's metric: context for it (what the method's attention path costs per block entry and per step)."""
    import torch

    import focus_inputs as fi
    from paper_2602_02159_amd.step import FocusDecoder
    dev = torch.device("cuda:0")
    w = fi.WORKLOADS["stack32k"]
    n_layers, l_dense = w.n_layers, w.probe_layer
    dec = FocusDecoder(n_layers, l_dense, 0, w.n_heads, w.head_dim, w.n_ctx, w.n_resp, w.n_gen, w.n_ctx, w.block, w.k_focus,
                       w.window, w.n_keep, w.n_sink, dev)
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed)
    for l in range(n_layers):
        for t in (dec.q_all[l], dec.k_all[l], dec.v_all[l], dec.q[l], dec.k_new[l], dec.v_new[l]):
            t.copy_(torch.randn(t.shape, generator=gen, device=dev, dtype=torch.float32))
    dec.conf.copy_(torch.rand(w.n_gen, generator=gen, device=dev))
    dec.capture()
    torch.cuda.synchronize()

    def timed(fn, reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps   # ms

    ms_entry = timed(dec.run_entry, 1)
    dec.run_step()
    ms_step = timed(dec.run_step, args.steps)
    n_sparse = sum(dec.is_sparse(l) for l in range(n_layers))
    print(json.dumps({"mode": "decoder", "workload": w.name, "layers": n_layers, "dense_layers_incl_probe": l_dense + 1,
                      "sparse_layers": n_sparse, "ms_block_entry": round(ms_entry, 2), "ms_per_step": round(ms_step, 4),
                      "steps_timed": args.steps, "launch": "two HIP graphs (block entry, step)",
                      "n_active": int(dec.counts.cpu()[1])}))
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
    ap.add_argument("--no-paper-shapes", action="store_true", help="skip the paper32k sparse-attention measurement (roofline_paper32k)")
    ap.add_argument("--parse-clock", metavar="DB", help="print the shader-clock table of a `rocprofv3 --pmc GRBM_GUI_ACTIVE` run of `--mode refresh`")
    ap.add_argument("--mode", default="bench", choices=["bench", "pmc", "refresh", "decoder"],
                    help="pmc: run a 1 GiB copy (calibration) and a few launches of every stage, nothing else; meant to be "
                         "run under `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE`.  refresh: the block-entry attention and a "
                         "plain 8192^3 bf16 product on normal-distributed and on all-zero inputs")
    ap.add_argument("--parse-pmc", nargs=2, metavar=("FETCH_DB", "WRITE_DB"),
                    help="turn the two rocprofv3 --pmc result databases of a `--mode pmc` run into profiles/hbm_traffic_<workload>.json")
    ap.add_argument("--parse-mfma", metavar="DB", help="print the MFMA utilisation table of a rocprofv3 --pmc database (see parse_mfma)")
    ap.add_argument("--parse-trace", metavar="DB", help="print the per-kernel table of a rocprofv3 --kernel-trace database")
    args = ap.parse_args()
    if args.parse_trace:
        return parse_trace(args.parse_trace)
    if args.parse_clock:
        return parse_clock(args.parse_clock)
    if args.parse_mfma:
        return parse_mfma(args.parse_mfma, args.workload)
    if args.parse_pmc:
        return parse_pmc(args.parse_pmc[0], args.parse_pmc[1], args.workload)
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path has no multi-GPU part); run with --gpus 1", file=sys.stderr)
        return 2

    if args.mode == "decoder":
        return decoder_mode(args)
    if args.mode == "refresh":
        return refresh_mode(args)

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

    def sync():
        torch.cuda.synchronize()

    # ---- inputs, generated on the device from the seeded counter-based streams; `sets` independent copies.
    # The block entry is played once per layer: focus_cache_refresh moves the newly computed states into the K/V cache
    # the step reads and emits the block means from the same pass.
    def build_steps(wl, n_sets, p_layer, s_ids):
        conf_ = fi.confidence(wl, dev)
        masked_ = fi.masked_all(wl, dev)
        objs = []
        for s in range(n_sets):
            ws_ = wl.with_(seed=wl.seed + 7919 * s)
            probe = fi.layer_qkv(ws_, p_layer, dev, which="qkv")
            layers, kbars = [], []
            for l in s_ids:
                q, k_new, v_new = fi.layer_qkv(ws_, l, dev)
                k_cache, v_cache = torch.empty_like(k_new), torch.empty_like(v_new)
                kbar = torch.empty((wl.n_heads, wl.n_blocks, wl.head_dim), dtype=torch.float32, device=dev)
                fb.cache_refresh(k_cache, v_cache, fb.make_shape(q, k_cache, v_cache, wl.n_ctx, wl.block), k_new, v_new, kbar)
                sync()
                del k_new, v_new
                layers.append((q, k_cache, v_cache))
                kbars.append(kbar)
            objs.append(FocusStep(conf_, masked_, probe, layers, wl.n_ctx, wl.block, wl.k_focus, wl.window, wl.n_keep, wl.n_sink,
                                  cached_means=True, kbars=kbars))
        return conf_, masked_, objs

    t0 = time.time()
    conf, masked, steps_obj = build_steps(w, args.sets, probe_layer, sparse_ids)
    sync()
    gen_s = time.time() - t0

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
        for stage in ("block_means", "block_partials", "block_scores_cached", "sparse_attn", "sparse_layer_cached", "dense_attn",
                      "find_sinks", "probe_layer", "select"):
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

    # ---- eager run once: results used for the parity check and the byte counts
    for st in steps_obj:
        st.run()
    sync()
    st0 = steps_obj[0]

    def attended_keys(st, wl):
        sinks = st.sink_idx.cpu().tolist()
        n_keys = []
        for b in st.bufs:
            rows = set(j for j in sinks if 0 <= j < wl.n_ctx)
            for blk in b["kept"].cpu().tolist():
                rows.update(range(blk * wl.block, min((blk + 1) * wl.block, wl.n_ctx)))
            n_keys.append(len(rows) + wl.n_resp)
        return float(np.mean(n_keys))

    mean_keys = attended_keys(st0, w)
    n_q = int(st0.counts.cpu()[1])
    H, d, L, M = w.n_heads, w.head_dim, w.n_kv, w.n_ctx
    n_b = w.n_blocks

    # ---- algorithmic bytes / flops per launch of each stage: what the method must move, not what an implementation
    # may add (the logits spilled, or K read a second time, while scoring the sinks are not counted)
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

    # ---- the timed region: exactly K steps (query selection, sinks, every sparse layer from the cached block means)
    ms_step = time_steps(steps_obj, args.steps, args.warmup)

    # ---- secondary timings (same run)
    def variant(objs_in, **kw):
        objs = []
        for st in objs_in:
            v = FocusStep.__new__(FocusStep)
            v.__dict__.update(st.__dict__)
            v._graph = None
            for key, val in kw.items():
                setattr(v, key, val)
            if use_graph:
                v.capture()
            objs.append(v)
        return objs

    few = max(5, args.steps // 5)
    ms_warm = time_steps(steps_obj[:1], args.steps, args.warmup)          # one input set only: whatever fits stays in the caches
    ms_recomputed = time_steps(variant(steps_obj, cached_means=False), few, 2)   # K scanned again in every layer and step
    ms_dense = time_steps(variant(steps_obj, dense=True), few, 2)                # the same layers, every block attended
    ms_probe = time_steps(variant(steps_obj, use_probe_layer=True), few, 2)      # sinks as a by-product of the probe layer's dense attention

    # launch floor: a chain of trivial kernels in one graph (what a launch costs before it does anything)
    tiny_buf = torch.zeros(64, device=dev)
    for _ in range(2):
        tiny_buf.zero_()
    sync()
    g_floor = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g_floor):
        for _ in range(64):
            tiny_buf.zero_()
    g_floor.replay()
    sync()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        g_floor.replay()
    e1.record()
    sync()
    launch_floor_us = e0.elapsed_time(e1) * 1e3 / 640

    # ---- per-stage durations with HIP events on the launch stream, back to back over all layers of all sets
    def time_stage(objs, stage, reps):
        n_launch = 0
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for st in objs:
            st.issue(stage)
        sync()
        e0.record()
        for _ in range(reps):
            for st in objs:
                st.issue(stage)
                n_launch += len(st.calls[stage])
        e1.record()
        sync()
        return e0.elapsed_time(e1) * 1e3 / n_launch  # microseconds per launch

    stages = {}
    per_step_count = {"select": 1, "find_sinks": 1, "block_means": 0, "block_partials": 0, "block_scores_cached": n_sparse,
                      "block_scores": 0, "sparse_attn": n_sparse, "dense_attn": 0, "sparse_layer": 0,
                      "sparse_layer_cached": n_sparse, "probe_layer": 0}
    for stage in ("select", "find_sinks", "block_means", "block_partials", "block_scores_cached", "block_scores", "sparse_attn", "dense_attn",
                  "sparse_layer_cached", "sparse_layer", "probe_layer"):
        us = time_stage(steps_obj, stage, args.kernel_reps)
        a = alg[stage]
        stages[stage] = {"us_per_launch": round(us, 3), "launches_per_step": per_step_count[stage],
                         "alg_bytes": int(a["bytes"]), "alg_flops": int(a["flops"]),
                         "GBps": round(a["bytes"] / us * 1e-3, 1), "TFLOPps": round(a["flops"] / us * 1e-6, 3),
                         "hbm_frac": round(a["bytes"] / us * 1e-3 / HBM_PEAK_GBS, 4)}
    stages["sparse_layer_cached"]["note"] = "the step's per-layer call: relevance from cached means, attention with Top-C inside, combine"
    stages["sparse_attn"]["note"] = "focus_sparse_attn alone (attention kernel + split combine), kept blocks given"
    stages["block_means"]["note"] = stages["block_partials"]["note"] = "K scan: once per block entry (Eq. 3), not part of the step"

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
    # dense comparison with ALL positions of the generation block as queries (what a decoder without the query selection of
    # Eq. 4 / Eq. 5 runs in every layer): every key, every query of the block; rotated over the layers of the two input sets
    all_q = torch.arange(w.n_gen, dtype=torch.int32, device=dev)
    all_counts = torch.tensor([w.n_gen, w.n_gen], dtype=torch.int32, device=dev)
    all_blocks = torch.arange(n_b, dtype=torch.int32, device=dev)
    out_all_q = torch.empty(H, w.n_gen, d, dtype=torch.bfloat16, device=dev)
    d2_layers = [lay for so in steps_obj for lay in so.layers]
    d2_shapes = [fb.make_shape(qq, kk, vv, M, w.block, out_all_q) for qq, kk, vv in d2_layers]
    d2_ws = torch.empty(fb.workspace_bytes(fb.FN_SPARSE_ATTN, d2_shapes[0], w.n_gen, n_b, 0), dtype=torch.uint8, device=dev)
    d2_rot = [0]

    def d2_call():
        i = d2_rot[0] % len(d2_layers)
        d2_rot[0] += 1
        qq, kk, vv = d2_layers[i]
        fb.sparse_attn(qq, all_q, all_counts, kk, vv, d2_shapes[i], all_blocks, n_b, None, 0, out_all_q, None, d2_ws)

    us = time_call(d2_call, reps=len(d2_layers), replays=4)
    db2 = 2 * L * H * d * 2 + 2 * w.n_gen * H * d * 2
    stages["dense_attn_all_block_queries"] = {
        "us_per_launch": round(us, 3), "launches_per_step": 0, "alg_bytes": db2, "alg_flops": 4 * w.n_gen * L * d * H,
        "GBps": round(db2 / us * 1e-3, 1), "TFLOPps": round(4 * w.n_gen * L * d * H / us * 1e-6, 3),
        "hbm_frac": round(db2 / us * 1e-3 / HBM_PEAK_GBS, 4),
        "note": f"dense attention of all {w.n_gen} positions of the generation block over every key, one layer"}
    del vl, k_cache, v_cache, kbar_r, d2_ws
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

    # ---- roofline of the step's dominant stage.  The step calls focus_sparse_layer; its attention part is timed through
    # focus_sparse_attn, which runs the same attention kernel (without the Top-C prologue) and the same combine kernel.
    in_step = ("select", "find_sinks", "block_scores_cached", "sparse_attn")
    share = {s: stages[s]["us_per_launch"] * per_step_count[s] for s in in_step}
    dom = max(share, key=share.get)
    ds = stages[dom]
    cap_q = st0.max_active                              # the launchers plan for the capacity of the active list
    qtw = 1 if cap_q <= 16 else (2 if cap_q <= 32 else 4)   # query tiles per workgroup they pick

    def attn_traffic(workload_name, qt):
        """HBM bytes of one focus_sparse_attn call (attention kernel: rows fetched + split partials written; combine: partials
        re-read + output written) from the stored rocprofv3 --pmc run of this script (--mode pmc, --parse-pmc)."""
        try:
            with open(PMC_FILE.format(workload_name)) as fh:
                pmc = json.load(fh)
            total = 0
            hit = False
            for name, v in pmc["kernels"].items():
                if f"sparse_attn_kernel<{d}, {qt}, 0>" in name:   # a name the dense comparison shares: the smallest dispatch is the sparse one
                    total += int(v["fetch_bytes_min"] + v["write_bytes_min"])
                    hit = True
                elif "attn_combine_kernel" in name:
                    total += int(v["fetch_bytes_min"] + v["write_bytes_min"])
            return total if hit else None
        except (OSError, KeyError, ValueError):
            return None

    kernel_names = {"sparse_attn": f"sparse_attn_kernel<{d}, {qtw}, 0> + attn_combine_kernel<{d}> (one focus_sparse_attn call; in the step the "
                                   f"attention kernel is the <{d}, {qtw}, 1> variant with the Top-C prologue)",
                    "find_sinks": f"qk_logits_kernel<{d}, {qtw}, {0 if qtw == 1 else 1}> and the rest of the sink chain",
                    "block_scores_cached": f"relevance_partial_kernel<{d}> + reduce_topk_kernel", "select": "select_queries_kernel"}
    traffic = attn_traffic(w.name, qtw) if dom == "sparse_attn" else None
    roofline = {"bound": "hbm", "kernel": kernel_names[dom], "stage": dom, "achieved": ds["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": ds["hbm_frac"], "traffic": traffic,
                "traffic_source": None if traffic is None else f"profiles/hbm_traffic_{w.name}.json: a separate rocprofv3 --pmc run of "
                                  "`bench.py --mode pmc` (FETCH_SIZE, WRITE_SIZE), not measured in this run",
                "us_per_launch": ds["us_per_launch"], "alg_bytes_per_launch": ds["alg_bytes"],
                "launches_per_step": per_step_count[dom], "launch_floor_us": round(launch_floor_us, 3)}

    step_bytes = alg["select"]["bytes"] + alg["find_sinks"]["bytes"] + n_sparse * alg["sparse_layer_cached"]["bytes"]
    step_flops = alg["find_sinks"]["flops"] + n_sparse * alg["sparse_layer_cached"]["flops"]
    dense_bytes = alg["select"]["bytes"] + alg["find_sinks"]["bytes"] + n_sparse * alg["dense_attn"]["bytes"]

    # ---- the sparse attention at the paper's own hyper-parameters (w = 8, block 64, alpha = 0.5, N_sink = 0.01 M): the one
    # sparse launch of the method that moves enough bytes (272 MB) to be bound by bandwidth rather than by latency
    roofline_paper = None
    if not args.no_paper_shapes and w.name == "stack32k":
        wp = fi.WORKLOADS["paper32k"]
        _, _, p_objs = build_steps(wp, 4, 0, [0])   # four copies rotated: 2.2 GB of K/V between reuses
        for st in p_objs:
            st.run()
        sync()
        keys_p = attended_keys(p_objs[0], wp)
        nq_p = int(p_objs[0].counts.cpu()[1])
        bytes_p = 2 * keys_p * wp.n_heads * wp.head_dim * 2 + 2 * nq_p * wp.n_heads * wp.head_dim * 2
        flops_p = 4 * nq_p * keys_p * wp.head_dim * wp.n_heads
        us_p = time_stage(p_objs, "sparse_attn", 8)
        us_pl = time_stage(p_objs, "sparse_layer_cached", 8)
        us_pd = time_stage(p_objs, "dense_attn", 4)
        us_ps = time_stage(p_objs, "find_sinks", 4)
        cap_p = p_objs[0].max_active
        qt_p = 1 if cap_p <= 16 else (2 if cap_p <= 32 else 4)
        tr_p = attn_traffic(wp.name, qt_p)
        roofline_paper = {"bound": "hbm", "workload": "paper32k", "stage": "sparse_attn",
                          "kernel": f"sparse_attn_kernel<{wp.head_dim}, {qt_p}, 0> + attn_combine_kernel<{wp.head_dim}> (one focus_sparse_attn call)",
                          "achieved": round(bytes_p / us_p * 1e-3, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                          "frac": round(bytes_p / us_p * 1e-3 / HBM_PEAK_GBS, 4), "traffic": tr_p,
                          "traffic_source": None if tr_p is None else "profiles/hbm_traffic_paper32k.json (separate rocprofv3 --pmc run)",
                          "us_per_launch": round(us_p, 3), "alg_bytes_per_launch": int(bytes_p), "TFLOPps": round(flops_p / us_p * 1e-6, 1),
                          "n_queries": nq_p, "mean_keys_attended": keys_p, "n_keep": wp.n_keep, "n_sink": wp.n_sink, "block": wp.block,
                          "us_sparse_layer_cached": round(us_pl, 3), "us_dense_attn_same_queries": round(us_pd, 3),
                          "us_find_sinks": round(us_ps, 3)}
        del p_objs
        torch.cuda.empty_cache()

    # ---- parity check + CPU baseline: the oracle on the probe layer and on every sparse layer of set 0
    cpu = None
    parity = None
    parity_ok = True
    if not args.no_cpu_baseline:
        from oracle import focus_oracle as fo
        from threadpoolctl import threadpool_info, threadpool_limits
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        to_np = lambda t: t.float().cpu().numpy()
        st0.release_graph()
        st0.run()
        sync()
        Qp, Kp = to_np(st0.probe[0]), to_np(st0.probe[1])
        conf_np = conf.cpu().numpy()
        cpu0 = time.process_time()
        t = time.perf_counter()
        focus_ref = fo.select_focus(conf_np, None, w.k_focus)
        active_ref = fo.expand_window(focus_ref, w.window, 0, w.n_gen)
        sinks_ref = fo.select_sinks(fo.sink_scores(Qp, active_ref, Kp), w.n_ctx, w.n_sink)
        t_once = time.perf_counter() - t
        cpu_busy = time.process_time() - cpu0
        t_layers, kept_ok, errs = 0.0, True, []
        first = None
        for i in range(n_sparse):           # one layer's tensors on the host at a time
            Q, K, V = (to_np(x) for x in st0.layers[i])
            if first is None:
                first = (Q, K, V)
            cpu0 = time.process_time()
            t = time.perf_counter()
            lay = fo.focus_layer(Q, K, V, focus_ref, active_ref, sinks_ref, w.n_ctx, w.block, w.n_keep)
            t_layers += time.perf_counter() - t
            cpu_busy += time.process_time() - cpu0
            kept_ok = kept_ok and st0.bufs[i]["kept"].cpu().tolist() == lay["blocks"].tolist()
            errs.append(np.abs(to_np(st0.bufs[i]["out"])[:, :n_q] - lay["out"]))   # rows past |I_active| are padding
        cpu_ms = (t_once + t_layers) * 1e3
        # the same oracle on one thread: the probe layer and one sparse layer, the layer time scaled to all of them
        with threadpool_limits(limits=1):
            t = time.perf_counter()
            fo.select_sinks(fo.sink_scores(Qp, active_ref, Kp), w.n_ctx, w.n_sink)
            t1_once = time.perf_counter() - t
            t = time.perf_counter()
            fo.focus_layer(*first, focus_ref, active_ref, sinks_ref, w.n_ctx, w.block, w.n_keep)
            t1_layer = time.perf_counter() - t
        # threads the oracle actually kept busy: CPU time over wall time (its per-head matrix products are too small for
        # the BLAS pool to spread, so this is close to one whatever the pool size)
        used = max(1, int(round(cpu_busy / max(t_once + t_layers, 1e-9))))
        cpu = {"value": round(cpu_ms, 1), "unit": "ms", "cores": used, "blas_pool_threads": int(cores), "kind": "oracle",
               "sample": f"the whole step on input set 0: query selection + sink identification on the probe layer and all {n_sparse} sparse "
                         "layers (block means, relevance, Top-C, attention), float64 numpy with its BLAS thread pool",
               "value_single_thread": round((t1_once + n_sparse * t1_layer) * 1e3, 1),
               "sample_single_thread": f"BLAS pool limited to one thread: the probe layer and 1 of the {n_sparse} sparse layers, "
                                       f"layer time scaled to {n_sparse}", "host_cpus": os.cpu_count()}
        parity = {
            "focus_idx": st0.focus_idx.cpu().tolist() == focus_ref.tolist(),
            "sink_idx": st0.sink_idx.cpu().tolist() == sinks_ref.tolist(),
            "kept_blocks": bool(kept_ok), "layers_checked": n_sparse,
            "attn_max_abs_err": float(max(e.max() for e in errs)), "attn_mean_abs_err": float(max(e.mean() for e in errs)),
        }
        parity_ok = parity["focus_idx"] and parity["sink_idx"] and parity["kept_blocks"] and \
            parity["attn_max_abs_err"] <= 2e-2 and parity["attn_mean_abs_err"] <= 2e-3
        parity["ok"] = bool(parity_ok)

    out = {
        "metric": "sparse-attn step latency at 32K ctx" if "32k" in w.name else f"sparse-attn step latency ({w.name})",
        "value": round(ms_step, 4), "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "layers_in_step": f"probe {probe_layer} + sparse {sparse_ids[0]}..{sparse_ids[-1]}",
                   "heads": H, "head_dim": d, "n_ctx": M, "n_resp": w.n_resp, "block": w.block, "n_queries": n_q,
                   "n_keep": w.n_keep, "n_sink": w.n_sink, "mean_keys_attended": mean_keys, "launch": "hip_graph" if use_graph else "eager",
                   "input_sets_rotated": args.sets, "block_means": "cached at block entry (emitted by focus_cache_refresh before the clock starts)",
                   "per_layer_call": "focus_sparse_layer with K_bar (relevance from the cached means, attention with Top-C inside, combine)"},
        "achieved_hbm_GBps": round(step_bytes / ms_step * 1e-6, 1), "achieved_TFLOPps": round(step_flops / ms_step * 1e-9, 3),
        "step_alg_bytes": int(step_bytes), "step_hbm_frac": round(step_bytes / ms_step * 1e-6 / HBM_PEAK_GBS, 4),
        "ms_per_step_warm_caches": round(ms_warm, 4),
        "ms_per_step_block_means_recomputed": round(ms_recomputed, 4),
        "ms_per_step_sinks_from_probe_layer": round(ms_probe, 4),
        # the probe layer is a dense layer the model runs in any case (Alg. 1: layers up to l_dense are dense): what the sinks
        # cost on top of it = probe-layer call - dense attention of the same queries, per launch
        "us_sinks_on_top_of_the_dense_probe_layer": round(stages["probe_layer"]["us_per_launch"] - stages["dense_attn"]["us_per_launch"], 3),
        "ms_per_step_dense_attention": round(ms_dense, 4),
        "dense_over_sparse": round(ms_dense / ms_step, 2),
        "dense_step_hbm_frac": round(dense_bytes / ms_dense * 1e-6 / HBM_PEAK_GBS, 4),
        "launch_floor_us": round(launch_floor_us, 3),
        "paper_speedup_context": ">29x end-to-end decoding speedup over vanilla at 32K on NVIDIA H200 (whole 8B model; not comparable)",
        "roofline": roofline,
        "roofline_paper32k": roofline_paper,
        # not part of the step: the one MFMA-bound launch of the method (block entry, every position attends to every key)
        "roofline_block_entry": None if "full_refresh_layer" not in stages else {
            "bound": "mfma", "kernel": f"refresh_attn_kernel<{d}, 1, 8>", "achieved": stages["full_refresh_layer"]["TFLOPps"],
            "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": stages["full_refresh_layer"]["mfma_frac"],
            "us_per_launch": stages["full_refresh_layer"]["us_per_launch"], "flops_per_launch": stages["full_refresh_layer"]["alg_flops"]},
        "stages": stages, "cpu_baseline": cpu, "parity_vs_oracle": parity, "input_gen_s": round(gen_s, 1),
    }
    print(json.dumps(out))
    if not parity_ok:
        print("bench.py: the timed buffers do not match the oracle", file=sys.stderr)
        return 3
    return 0


if __name__ == "__main__":
    sys.exit(main())
