#!/usr/bin/env python3
"""Benchmark of the LSP hot path on one MI355X.

A step is one pass of the whole hot path over the 6.7B-style layer stack (benchmark configuration 4):
32 layers x {down 11008x4096, gate/up 4096x11008, o/v/k/q 4096x4096}, bf16, r = 512, d = 8,
visited layer by layer in backward order; every matrix gets one lsp_compress_planned
(S = P^T G Q) and one lsp_decompress_apply (W -= P S Q^T).  The seven matrices of a layer are
independent: by default they go out as one grouped call per kernel family
(lsp_compress_planned_grouped, lsp_decompress_apply_grouped), all on ONE stream, layer after layer (the
named workload); --grouped 0 issues one call per matrix instead, --streams N deals the layers to N HIP
streams (default priority, joined at the end of the step).  The reported value is the one-stream step; the
same step on two streams is timed beside it and labelled.  The roofline legs time each kernel family alone
on one stream: the grouped calls of the step back to back, and (reported beside them) one call per matrix.
All inputs are resident in HBM before the timed region; all 224 G / W / S / projector buffers are distinct.

Prints ONE JSON line: throughput in algorithmic GB/s (the bytes the method must move: G once for
compress, W read and written for decompress-apply, plus the projector arrays and S) with a roofline object for the dominant kernel and the CPU oracle timed on a bounded
sample beside it.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X published HBM3E bandwidth


def algorithmic_bytes(m, n, r, d, sz):
    comp = m * n * sz + (m + n) * d * 8 + r * r * 4
    deco = 2 * m * n * sz + (m + n) * d * 8 + r * r * 4
    return comp, deco


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--layers", type=int, default=32, help="layers of the stack (32 = the named workload)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--grouped", type=int, default=1,
                    help="1: one grouped call per layer and kernel family; 0: one call per matrix")
    ap.add_argument("--streams", type=int, default=1,
                    help="HIP streams the layers are dealt to (default priority; joined at step end); 1 = the named workload")
    ap.add_argument("--dense-ablation", action="store_true",
                    help="instead of the step: the sparse compress path at d = 2..16 against the same contraction "
                         "with dense bf16 projectors through the vendor GEMM (prints its own JSON line)")
    ap.add_argument("--other-configs", action="store_true",
                    help="instead of the step: one-call timings of the other benchmark configurations and of the "
                         "paper-sized subspaces (prints its own JSON line)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this path is single-GPU by construction (no collectives are built); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import lsp_synth as syn
    import paper_2406_10181_amd as L

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.current_stream()
    if args.dense_ablation:
        print(json.dumps(dense_ablation(torch, syn, L, dev, stream)), flush=True)
        return
    if args.other_configs:
        print(json.dumps(other_configs(torch, syn, L, dev, stream)), flush=True)
        return
    r, d, dtype, code, sz = 512, 8, "bf16", syn.DTYPE_CODE["bf16"], 2

    # ------------------------------------------------------------------ inputs, resident in HBM
    t0 = time.time()
    plan_ms = {}    # shape -> wall times of lsp_plan_build (a set-up call, once per projector refresh)
    mats = []       # backward order: layer L-1 .. 0; within a layer: down, gate, up, o, v, k, q
    ws_bytes = 0
    gen = torch.Generator(device=dev)
    for layer in range(args.layers - 1, -1, -1):
        for which, (name, m, n) in enumerate(syn.LAYER_67B):
            seed = 4000 + layer * 7 + which
            gen.manual_seed(seed)
            G = (torch.randn(m, n, device=dev, generator=gen, dtype=torch.float32) * 1e-3).to(torch.bfloat16)
            W = (torch.randn(m, n, device=dev, generator=gen, dtype=torch.float32) * 0.02).to(torch.bfloat16)
            S_upd = torch.randn(r, r, device=dev, generator=gen, dtype=torch.float32) * 1e-3
            rng = np.random.default_rng(seed)
            P_idx, P_val = syn.ell_projector(m, r, d, rng, "uniform")
            Q_idx, Q_val = syn.ell_projector(n, r, d, rng, "uniform")
            e = dict(name=f"L{layer}_{name}", m=m, n=n, G=G, W=W, S_upd=S_upd,
                     S=torch.empty(r, r, device=dev, dtype=torch.float32),
                     P_idx=torch.from_numpy(P_idx).to(dev), P_val=torch.from_numpy(P_val).to(dev),
                     Q_idx=torch.from_numpy(Q_idx).to(dev), Q_val=torch.from_numpy(Q_val).to(dev))
            # the expand side (decompress-apply, estimation bias) gets the copy of Q whose rows are ordered against
            # LDS bank conflicts: the same projector, prepared once per change of projectors like the plan
            qi, qv = np.empty_like(Q_idx), np.empty_like(Q_val)
            L.lsp_projector_reorder_host(Q_idx, Q_val, n, d, r, qi, qv)
            e["Qx_idx"], e["Qx_val"] = torch.from_numpy(qi).to(dev), torch.from_numpy(qv).to(dev)
            pbytes = L.lsp_plan_bytes(m, n, r, d)
            e["plan"] = torch.empty(pbytes, dtype=torch.uint8, device=dev)
            torch.cuda.synchronize()
            tp = time.perf_counter()
            L.lsp_plan_build(e["P_idx"], e["P_val"], e["Q_idx"], e["Q_val"], m, n, r, d, e["plan"], pbytes, stream)
            plan_ms.setdefault(f"{m}x{n}", []).append((time.perf_counter() - tp) * 1e3)      # the call is synchronous
            ws_bytes = max(ws_bytes, L.lsp_compress_planned_workspace_bytes(m, n, r, d))
            e["cb"], e["db"] = algorithmic_bytes(m, n, r, d, sz)
            mats.append(e)
    nstreams = max(1, args.streams)
    nlanes = max(2, nstreams)                                                          # a second stream for the labelled two-stream leg
    lanes = [stream] + [torch.cuda.Stream(device=dev) for _ in range(nlanes - 1)]     # default priority
    wss = [torch.empty(ws_bytes, dtype=torch.uint8, device=dev) for _ in lanes]       # one workspace per stream
    fork = torch.cuda.Event()
    joins = [torch.cuda.Event() for _ in lanes]
    torch.cuda.synchronize()
    setup_s = time.time() - t0

    def compress_all(ms, ns=1):
        for k, e in enumerate(ms):
            q = k % ns
            L.lsp_compress_planned(e["G"], e["plan"], e["m"], e["n"], r, d, e["S"], code, wss[q], ws_bytes, lanes[q])

    def decompress_all(ms, ns=1):
        for k, e in enumerate(ms):
            q = k % ns
            L.lsp_decompress_apply(e["W"], e["S_upd"], e["P_idx"], e["P_val"], e["Qx_idx"], e["Qx_val"],
                                   e["m"], e["n"], r, d, code, lanes[q])

    # grouped mode: the seven matrices of a layer in one call (own S and workspace each); layers
    # alternate over the streams
    layers = [mats[k:k + 7] for k in range(0, len(mats), 7)]
    gws = [[torch.empty(L.lsp_compress_planned_workspace_bytes(e["m"], e["n"], r, d), dtype=torch.uint8, device=dev)
            for e in layers[0]] for _ in lanes]
    citems = [L.compress_items([(e["G"], e["plan"], e["S"], gws[li % nlanes][k], gws[li % nlanes][k].numel(),
                                 e["m"], e["n"]) for k, e in enumerate(ly)]) for li, ly in enumerate(layers)]
    aitems = [L.apply_items([(e["W"], e["S_upd"], e["P_idx"], e["P_val"], e["Qx_idx"], e["Qx_val"], e["m"], e["n"])
                             for e in ly]) for ly in layers]

    def step_grouped(ns=None):
        ns = nstreams if ns is None else ns
        for li in range(len(layers)):
            q = lanes[li % ns]
            L.lsp_compress_planned_grouped(citems[li], 7, r, d, code, q)
            L.lsp_decompress_apply_grouped(aitems[li], 7, r, d, code, q)

    def grouped_pass(which, ns=None):
        ns = nstreams if ns is None else ns
        for li in range(len(layers)):
            q = lanes[li % ns]
            if which == "c":
                L.lsp_compress_planned_grouped(citems[li], 7, r, d, code, q)
            else:
                L.lsp_decompress_apply_grouped(aitems[li], 7, r, d, code, q)

    def forked(fn, ns=None):
        # side streams start after everything already queued on the main stream and are joined
        # back into it, so events recorded on the main stream bracket all the work
        ns = nstreams if ns is None else ns
        if ns == 1:
            return fn()
        fork.record(stream)
        for s in lanes[1:ns]:
            s.wait_event(fork)
        fn()
        for s, ev in zip(lanes[1:ns], joins[1:ns]):
            ev.record(s)
            stream.wait_event(ev)

    def step_body(ns=None):
        # layer by layer: the layer's compress calls, then its decompress-apply calls; a matrix
        # stays on one stream, so its two calls are ordered
        ns = nstreams if ns is None else ns
        for k in range(0, len(mats), 7):
            compress_all(mats[k:k + 7], ns)
            decompress_all(mats[k:k + 7], ns)

    def step():
        forked(step_grouped if args.grouped else step_body)

    def timed(fn, reps, each=None):
        """ms per repetition over `reps` back-to-back repetitions between two events on the working stream;
        each: a list that receives the individual repetitions' times (events between them, no host sync)."""
        torch.cuda.synchronize()
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
        marks[0].record(stream)
        for k in range(reps):
            fn()
            if each is not None or k == reps - 1:
                marks[k + 1].record(stream)
        torch.cuda.synchronize()
        if each is not None:
            each.extend(marks[k].elapsed_time(marks[k + 1]) for k in range(reps))
        return marks[0].elapsed_time(marks[reps]) / reps

    for _ in range(args.warmup):
        step()
    step_times = []
    ms_step = timed(step, args.steps, step_times)
    # the same step with the layers alternating over two streams (not the named workload: reported beside it)
    step2 = lambda: forked(lambda: step_grouped(2) if args.grouped else step_body(2), 2)
    step2()
    ms_step2 = timed(step2, max(3, min(args.steps, 10)))
    # per-kernel passes for the roofline: one stream, launches back to back, so the time per launch
    # is the kernel's own duration (same buffers, still cold: 26 GB is swept between two visits)
    sub = max(3, min(args.steps, 10))
    ms_comp = timed(lambda: compress_all(mats), sub)
    ms_deco = timed(lambda: decompress_all(mats), sub)

    ms_gcomp = timed(lambda: forked(lambda: grouped_pass("c", 2), 2), sub)
    ms_gdeco = timed(lambda: forked(lambda: grouped_pass("d", 2), 2), sub)
    # roofline legs: the grouped launches of the step, back to back on one stream, so that the time
    # per launch is the kernels' own duration
    ms_gcomp1 = timed(lambda: grouped_pass("c", 1), sub)
    ms_gdeco1 = timed(lambda: grouped_pass("d", 1), sub)

    # widening beyond the step: the estimation-bias pass (Def. 2) over every gradient of the stack,
    # one call per matrix on one stream; S holds P^T G Q from the compress passes above
    bias_ws_bytes = max(L.lsp_estimation_bias_workspace_bytes(e["m"], e["n"], r, d) for e in mats)
    bias_ws = torch.empty(bias_ws_bytes, dtype=torch.uint8, device=dev)
    bias_out = torch.zeros(3, dtype=torch.float32, device=dev)

    def bias_all():
        for e in mats:
            L.lsp_estimation_bias(e["G"], e["S"], e["P_idx"], e["P_val"], e["Qx_idx"], e["Qx_val"], e["m"], e["n"], r, d,
                                  bias_out, bias_ws, bias_ws_bytes, code, stream)
    ms_bias = timed(bias_all, sub)
    bbytes = sum(e["cb"] for e in mats)             # one read of G, the projector arrays and S: as for compress

    # one iteration of projector fitting on the GPU (MaybeUpdate, Alg. 1 / Eq. 2): new values into the plan, then the
    # gradient of 1/2 ||P P^T G Q Q^T - G||_F^2 with respect to the stored values, one 4096 x 4096 matrix
    fe = [e for e in mats if e["m"] == 4096 and e["n"] == 4096][0]
    fg_bytes = L.lsp_bias_gradient_workspace_bytes(4096, 4096, r, d)
    fg_ws = torch.empty(fg_bytes, dtype=torch.uint8, device=dev)
    fg_P = torch.empty(4096, d, dtype=torch.float32, device=dev)
    fg_Q = torch.empty(4096, d, dtype=torch.float32, device=dev)

    def fit_iteration():
        L.lsp_plan_refresh_values(fe["plan"], fe["P_val"], fe["Q_val"], 4096, 4096, r, d, stream)
        L.lsp_bias_gradient(fe["G"], fe["plan"], fe["P_idx"], fe["P_val"], fe["Q_idx"], fe["Q_val"], 4096, 4096, r, d,
                            fg_P, fg_Q, fg_ws, fg_bytes, code, stream)
    fit_iteration()
    ms_fit = timed(fit_iteration, 10)
    ms_refresh = timed(lambda: L.lsp_plan_refresh_values(fe["plan"], fe["P_val"], fe["Q_val"], 4096, 4096, r, d, stream), 10)

    # state re-projection after a change of projectors (MaybeUpdate, Alg. 1): one 4096 x 4096 matrix, the
    # projectors of two consecutive entries of the stack standing in for (new, previous)
    sq = [e for e in mats if e["m"] == 4096 and e["n"] == 4096][:2]
    rp_bytes = L.lsp_reproject_state_workspace_bytes(r)
    rp_ws = torch.empty(rp_bytes, dtype=torch.uint8, device=dev)
    rp_M = torch.randn(r, r, device=dev, dtype=torch.float32)
    rp_V = torch.rand(r, r, device=dev, dtype=torch.float32)
    ms_rep = timed(lambda: L.lsp_reproject_state(sq[0]["P_idx"], sq[0]["P_val"], sq[1]["P_idx"], sq[1]["P_val"],
                                                 sq[0]["Q_idx"], sq[0]["Q_val"], sq[1]["Q_idx"], sq[1]["Q_val"],
                                                 4096, 4096, r, d, rp_M, rp_V, rp_ws, rp_bytes, stream), 10)

    # what a kernel with nothing but the stream in it reaches here: a read-only pass and y -= c over 1 GiB (fp32),
    # same run, same stream; the buffer is four times the memory-side cache, so every pass comes from HBM
    probe_bytes = 1 << 30
    probe = torch.zeros(probe_bytes // 4, dtype=torch.float32, device=dev)
    pws_bytes = L.lsp_hbm_probe_workspace_bytes(probe_bytes)
    pws = torch.empty(pws_bytes, dtype=torch.uint8, device=dev)
    L.lsp_hbm_probe_read(probe, probe_bytes, pws, pws_bytes, stream)
    L.lsp_hbm_probe_rmw(probe, probe_bytes, 1.0, stream)
    ms_pread = timed(lambda: L.lsp_hbm_probe_read(probe, probe_bytes, pws, pws_bytes, stream), 10)
    ms_prmw = timed(lambda: L.lsp_hbm_probe_rmw(probe, probe_bytes, 1.0, stream), 10)
    read_gbs = probe_bytes / (ms_pread * 1e-3) / 1e9
    rmw_gbs = 2 * probe_bytes / (ms_prmw * 1e-3) / 1e9
    del probe

    # the plan build as the per-refresh loop would issue it: asynchronous, scratch allocated once, timed by events
    plan_async_us = {}
    for e in layers[0]:
        key = f'{e["m"]}x{e["n"]}'
        if key in plan_async_us:
            continue
        pb_bytes = L.lsp_plan_bytes(e["m"], e["n"], r, d)
        pw_bytes = L.lsp_plan_build_workspace_bytes(e["m"], e["n"], r, d)
        tmp_plan = torch.empty(pb_bytes, dtype=torch.uint8, device=dev)
        pw = torch.empty(pw_bytes, dtype=torch.uint8, device=dev)
        build = lambda: L.lsp_plan_build_async(e["P_idx"], e["P_val"], e["Q_idx"], e["Q_val"], e["m"], e["n"], r, d, tmp_plan,
                                               pb_bytes, pw, pw_bytes, None, stream)
        build()
        plan_async_us[key] = round(timed(build, 10) * 1e3, 1)
        assert torch.equal(tmp_plan, e["plan"]), "a rebuilt plan must equal the plan in use"
        del tmp_plan, pw

    # the call shape of the benchmark spec, lsp_compress on raw ELL arrays (plan built on the device inside the
    # call, every call), on the seven matrices of the first layer visited
    raw_ws = torch.empty(max(L.lsp_compress_workspace_bytes(e["m"], e["n"], r, d) for e in layers[0]), dtype=torch.uint8, device=dev)

    def raw_layer():
        for e in layers[0]:
            L.lsp_compress(e["G"], e["P_idx"], e["P_val"], e["Q_idx"], e["Q_val"], e["m"], e["n"], r, d, e["S"], code,
                           raw_ws, raw_ws.numel(), stream)
    raw_layer()
    ms_raw = timed(raw_layer, 3)
    raw_gbs = sum(e["cb"] for e in layers[0]) / (ms_raw * 1e-3) / 1e9

    cbytes = sum(e["cb"] for e in mats)
    dbytes = sum(e["db"] for e in mats)
    cflop = sum(2 * e["m"] * e["n"] * d + 2 * e["m"] * d * r for e in mats)
    value = (cbytes + dbytes) / (ms_step * 1e-3) / 1e9
    comp_gbs = cbytes / (ms_comp * 1e-3) / 1e9
    deco_gbs = dbytes / (ms_deco * 1e-3) / 1e9

    def traffic_of(fname, key):
        tpath = os.path.join(ROOT, "profiles", fname)
        try:
            return json.load(open(tpath)).get(key)
        except Exception:
            return None
    traffic_c = traffic_of("traffic_compress_cfg4.json", "hbm_bytes_per_launch")
    traffic_d = traffic_of("traffic_decompress_cfg4.json", "hbm_bytes_per_launch")
    traffic_gc = traffic_of("traffic_compress_cfg4.json", "hbm_bytes_per_grouped_launch")
    traffic_gd = traffic_of("traffic_decompress_cfg4.json", "hbm_bytes_per_grouped_launch")

    nlaunch = len(mats)
    out = {
        "metric": "compress+decompress GB/s per layer and % of MI355X HBM peak",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"cfg4: 6.7B-style stack, {args.layers} layers x 7 matrices, bf16 G/W, r=512, d=8, "
                               f"uniform projector columns, backward order, {nstreams} stream(s), " +
                               ("one grouped call per layer and kernel family" if args.grouped else "one call per matrix"),
                   "storage": "bf16", "accumulate": "f32", "matrices": nlaunch, "streams": nstreams, "grouped": bool(args.grouped),
                   "algorithmic_GB_per_step": round((cbytes + dbytes) / 1e9, 3)},
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "per_layer_us": round(ms_step * 1e3 / args.layers, 2),
        "ms_per_step_median": round(float(np.median(step_times)), 4), "ms_per_step_min": round(min(step_times), 4),
        # plain streaming kernels of this library over 1 GiB in the same run: the practical ceilings of the two calls
        "achievable_read_GBs": round(read_gbs, 1), "achievable_rmw_GBs": round(rmw_gbs, 1),
        # time the two plain streams would need for the step's algorithmic bytes, over the step's time
        "pct_of_achievable": round(100.0 * (cbytes / read_gbs + dbytes / rmw_gbs) / 1e9 / (ms_step * 1e-3), 2),
        # not the named workload: the same step with the layers alternating over two HIP streams
        "two_streams": {"ms_per_step": round(ms_step2, 4), "GB/s": round((cbytes + dbytes) / (ms_step2 * 1e-3) / 1e9, 1),
                        "pct_of_hbm_peak": round(100.0 * (cbytes + dbytes) / (ms_step2 * 1e-3) / 1e9 / HBM_PEAK_GBS, 2)},
        # set-up side, outside the step: lsp_plan_build once per projector refresh (synchronous form: host wall time with
        # its scratch allocation and the wait; asynchronous form: device time by events), and the raw-ELL entry that
        # builds its plan inside every call
        "plan_build_ms_per_matrix": {k: round(float(np.median(v)), 2) for k, v in plan_ms.items()},
        "plan_build_async_us_per_matrix": plan_async_us,
        "raw_lsp_compress": {"GB/s": round(raw_gbs, 1), "pct_of_hbm_peak": round(100 * raw_gbs / HBM_PEAK_GBS, 2),
                             "us_per_layer": round(ms_raw * 1e3, 1), "sample": "the seven matrices of one layer, one call each"},
        "compress": {"GB/s": round(comp_gbs, 1), "pct_of_hbm_peak": round(100 * comp_gbs / HBM_PEAK_GBS, 2),
                     "ms_per_pass": round(ms_comp, 4)},
        "decompress_apply": {"GB/s": round(deco_gbs, 1), "pct_of_hbm_peak": round(100 * deco_gbs / HBM_PEAK_GBS, 2),
                             "ms_per_pass": round(ms_deco, 4)},
        # the same two passes issued as in the step (grouped calls on the streams)
        "grouped": {"compress_ms_per_pass": round(ms_gcomp, 4), "compress_GB/s": round(cbytes / (ms_gcomp * 1e-3) / 1e9, 1),
                    "decompress_ms_per_pass": round(ms_gdeco, 4),
                    "decompress_GB/s": round(dbytes / (ms_gdeco * 1e-3) / 1e9, 1)},
        # dominant by GPU time: the two kernels of one grouped compress call (seven matrices), timed
        # together (one API call) on one stream
        "roofline": {"kernel": "k_compress_gq16<bf16> + k_compress_pt8 (one lsp_compress_planned_grouped call, 7 matrices)",
                     "bound": "hbm", "achieved": round(cbytes / (ms_gcomp1 * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(cbytes / (ms_gcomp1 * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                     "traffic": traffic_gc, "traffic_source": "profiles/traffic_compress_cfg4.json (rocprofv3 --pmc runs, not live)",
                     # the same launches against the vector-ALU roofline (useful flop only: one FMA per stored
                     # projector entry and element, 2 m n d + 2 m d r per matrix; widening bf16 is not counted)
                     "alu": {"TFLOP/s": round(cflop / (ms_gcomp1 * 1e-3) / 1e12, 2), "peak_fp32_vector_TFLOP/s": 157.3,
                             "frac": round(cflop / (ms_gcomp1 * 1e-3) / 1e12 / 157.3, 4)},
                     "launches": len(layers), "avg_launch_us": round(ms_gcomp1 * 1e3 / len(layers), 2),
                     "algorithmic_bytes_per_launch_avg": int(cbytes / len(layers)),
                     "per_matrix_calls": {"achieved": round(comp_gbs, 1), "frac": round(comp_gbs / HBM_PEAK_GBS, 4),
                                          "avg_launch_us": round(ms_comp * 1e3 / nlaunch, 2), "traffic": traffic_c}},
        "roofline_decompress": {"kernel": "k_decompress<bf16,d=8,r<=512> (one lsp_decompress_apply_grouped call, 7 matrices)",
                                "bound": "hbm", "achieved": round(dbytes / (ms_gdeco1 * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBS,
                                "unit": "GB/s", "frac": round(dbytes / (ms_gdeco1 * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                                "traffic": traffic_gd, "traffic_source": "profiles/traffic_decompress_cfg4.json (rocprofv3 --pmc runs, not live)",
                                "launches": len(layers), "avg_launch_us": round(ms_gdeco1 * 1e3 / len(layers), 2),
                                "algorithmic_bytes_per_launch_avg": int(dbytes / len(layers)),
                                "per_matrix_calls": {"achieved": round(deco_gbs, 1), "frac": round(deco_gbs / HBM_PEAK_GBS, 4),
                                                     "avg_launch_us": round(ms_deco * 1e3 / nlaunch, 2), "traffic": traffic_d}},
        # next row beyond the step (not part of `value`): the bias pass of Def. 2, one call per matrix
        "estimation_bias": {"kernel": "k_decompress<..., NORMS> + k_bias_finish (one lsp_estimation_bias call per matrix)",
                            "ms_per_pass": round(ms_bias, 4), "GB/s": round(bbytes / (ms_bias * 1e-3) / 1e9, 1),
                            "frac_of_hbm_peak": round(bbytes / (ms_bias * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                            "avg_call_us": round(ms_bias * 1e3 / nlaunch, 2)},
        # once per change of projectors: 4 dense r x r x r products on the matrix cores (fp32) + 2 sparse-sparse ones
        "reproject_state": {"kernel": "k_gram (both pairs) + k_gemm_rr4 x2, two products each (one lsp_reproject_state call, 4096 x 4096, r=512, d=8)",
                            "us_per_call": round(ms_rep * 1e3, 1), "bound": "mfma", "dense_flop": 8 * r ** 3,
                            "TFLOP/s": round(8 * r ** 3 / (ms_rep * 1e-3) / 1e12, 2), "peak_fp32_TFLOP/s": 157.3},
        # one fitting iteration on a 4096 x 4096 matrix: values-only plan refresh + gradient of the bias loss (G is
        # streamed twice: 2 x 33.6 MB algorithmic)
        "fitting_gradient": {"kernel": "k_plan_refresh + compress kernels + k_gram + k_gemm_rr4 x2 (five products) + k_gather_rows + k_grad_left/right "
                                       "(lsp_plan_refresh_values + lsp_bias_gradient, 4096 x 4096, r=512, d=8)",
                             "us_per_iteration": round(ms_fit * 1e3, 1), "plan_refresh_us": round(ms_refresh * 1e3, 1),
                             "GB/s_on_two_reads_of_G": round(2 * 4096 * 4096 * sz / (ms_fit * 1e-3) / 1e9, 1)},
        "setup_s": round(setup_s, 1),
    }

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(syn, r, d)
    print(json.dumps(out), flush=True)


def other_configs(torch, syn, L, dev, stream):
    """One lsp_compress_planned and one lsp_decompress_apply call per matrix, on one stream, for the shapes of the
    benchmark configurations other than the timed one and for the subspace sizes the paper trained with; uniform
    projector columns except for the wide sweep (bounded Zipf(1.1) columns in both projectors, as that configuration
    is specified), buffers rotating so that G / W come from HBM.  Times in us per call; percentages are the
    call's algorithmic bytes per second over the 8 TB/s HBM peak."""
    cases = [("cfg2", "f16", 2048, 2048, 256, 4, "uniform"), ("cfg3", "f16", 2048, 8192, 512, 4, "uniform"),
             ("cfg3", "f16", 8192, 2048, 512, 4, "uniform")]
    # the wide sweep as specified: both projectors' columns drawn from the bounded Zipf(1.1) distribution
    cases += [("cfg5 zipf", "bf16", 4096, 16384, r, d, "zipf") for r in (256, 512, 1024) for d in (2, 4, 8, 16)]
    cases += [("cfg5 shape, uniform columns", "bf16", 4096, 16384, 512, 8, "uniform")]
    cases += [("fp32", "f32", 4096, 4096, 512, 8, "uniform"), ("paper-sized subspace", "bf16", 4096, 4096, 2048, 8, "uniform"),
              ("paper-sized subspace", "f16", 2048, 2048, 1280, 4, "uniform")]
    tdt = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}
    rows = []
    for name, dt, m, n, r, d, dist in cases:
        code, esz = syn.DTYPE_CODE[dt], (4 if dt == "f32" else 2)
        nbuf = max(3, min(12, int(1.5e9 // (m * n * esz))))
        rng = np.random.default_rng(5000 + r + d if dist == "zipf" else 1)
        P_idx, P_val = syn.ell_projector(m, r, d, rng, dist)
        Q_idx, Q_val = syn.ell_projector(n, r, d, rng, dist)
        qi, qv = np.empty_like(Q_idx), np.empty_like(Q_val)
        L.lsp_projector_reorder_host(Q_idx, Q_val, n, d, r, qi, qv)          # the expand side gets the reordered copy of Q
        Qx_idx, Qx_val = torch.from_numpy(qi).to(dev), torch.from_numpy(qv).to(dev)
        P_idx, P_val, Q_idx, Q_val = [torch.from_numpy(x).to(dev) for x in (P_idx, P_val, Q_idx, Q_val)]
        Gs = [(torch.randn(m, n, device=dev) * 1e-3).to(tdt[dt]) for _ in range(nbuf)]
        S = torch.empty(r, r, device=dev)
        Su = torch.randn(r, r, device=dev) * 1e-3
        pbytes = L.lsp_plan_bytes(m, n, r, d)
        plan = torch.empty(pbytes, dtype=torch.uint8, device=dev)
        planned = L.lsp_plan_build(P_idx, P_val, Q_idx, Q_val, m, n, r, d, plan, pbytes, stream, check=False) == 0
        wb = max(L.lsp_compress_planned_workspace_bytes(m, n, r, d), L.lsp_compress_workspace_bytes(m, n, r, d))
        ws = torch.empty(wb, dtype=torch.uint8, device=dev)
        cb, db = algorithmic_bytes(m, n, r, d, esz)

        def run(fn, reps=3):
            for G in Gs[:2]:
                fn(G)
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            for _ in range(reps):
                for G in Gs:
                    fn(G)
            b.record(stream)
            torch.cuda.synchronize()
            return a.elapsed_time(b) * 1e3 / (reps * nbuf)
        if planned:
            tc = run(lambda G: L.lsp_compress_planned(G, plan, m, n, r, d, S, code, ws, wb, stream))
        else:   # columns too uneven for a plan (LSP_ERR_SKEW): the raw entry is the documented way
            tc = run(lambda G: L.lsp_compress(G, P_idx, P_val, Q_idx, Q_val, m, n, r, d, S, code, ws, wb, stream))
        td = run(lambda G: L.lsp_decompress_apply(G, Su, P_idx, P_val, Qx_idx, Qx_val, m, n, r, d, code, stream))
        rows.append({"config": name, "dtype": dt, "m": m, "n": n, "r": r, "d": d, "columns": dist,
                     "compress_entry": "lsp_compress_planned" if planned else "lsp_compress (raw; plan refused: skew)",
                     "compress_us": round(tc, 1), "compress_pct_of_hbm_peak": round(cb / tc / 1e3 / HBM_PEAK_GBS * 100, 1),
                     "decompress_us": round(td, 1), "decompress_pct_of_hbm_peak": round(db / td / 1e3 / HBM_PEAK_GBS * 100, 1)})
        del Gs, plan, ws
    return {"what": "one call per matrix on one stream, other configurations", "unit": "us per call", "rows": rows}


def dense_ablation(torch, syn, L, dev, stream):
    """Where does the sparse gather lose to a real contraction?  S = P^T G Q on config-4 shapes (bf16, r = 512):
    the library's sparse path (lsp_compress_planned) at d = 2, 4, 8, 16 entries per projector row, against
    T = G Qd, S = Pd^T T with the projectors densified and rounded to bf16, run on the matrix cores twice: by the
    library's own kernels (lsp_compress_dense: v_mfma_f32_32x32x16_bf16) and, as a second yardstick, by the vendor
    GEMM (torch.matmul).  bf16 projector values (8 significant bits) put the dense form outside the 1e-3 parity
    bar, which the reported error shows.  Buffers rotate so that G comes from HBM in all legs."""
    r, code, nbuf, reps = 512, syn.DTYPE_CODE["bf16"], 8, 3
    rows = []

    def timed(fn, Gs):
        for G in Gs[:2]:
            fn(G)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        for _ in range(reps):
            for G in Gs:
                fn(G)
        b.record(stream)
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e3 / (reps * len(Gs))          # us per call

    for (m, n) in ((4096, 4096), (4096, 11008)):
        gen = torch.Generator(device=dev)
        gen.manual_seed(7000 + n)
        Gs = [(torch.randn(m, n, device=dev, generator=gen, dtype=torch.float32) * 1e-3).to(torch.bfloat16)
              for _ in range(nbuf)]
        for d in (2, 4, 8, 16):
            rng = np.random.default_rng(7100 + n + d)
            P_idx, P_val = syn.ell_projector(m, r, d, rng, "uniform")
            Q_idx, Q_val = syn.ell_projector(n, r, d, rng, "uniform")
            tP_idx, tP_val, tQ_idx, tQ_val = [torch.from_numpy(x).to(dev) for x in (P_idx, P_val, Q_idx, Q_val)]
            pbytes = L.lsp_plan_bytes(m, n, r, d)
            plan = torch.empty(pbytes, dtype=torch.uint8, device=dev)
            L.lsp_plan_build(tP_idx, tP_val, tQ_idx, tQ_val, m, n, r, d, plan, pbytes, stream)
            wb = L.lsp_compress_planned_workspace_bytes(m, n, r, d)
            ws = torch.empty(wb, dtype=torch.uint8, device=dev)
            S = torch.empty(r, r, device=dev, dtype=torch.float32)
            t_sparse = timed(lambda G: L.lsp_compress_planned(G, plan, m, n, r, d, S, code, ws, wb, stream), Gs)
            S_sparse = S.clone()
            # dense projectors, rounded to bf16 (duplicates of a row add up first)
            Pd = torch.zeros(m, r, device=dev, dtype=torch.float32)
            Qd = torch.zeros(n, r, device=dev, dtype=torch.float32)
            Pd.scatter_add_(1, tP_idx.long(), tP_val)
            Qd.scatter_add_(1, tQ_idx.long(), tQ_val)
            Pdt = Pd.t().contiguous().to(torch.bfloat16)
            Qdb = Qd.to(torch.bfloat16)
            out = {}

            def dense(G):
                out["S"] = torch.matmul(Pdt, torch.matmul(G, Qdb))
            t_dense = timed(dense, Gs)
            Qdt = Qd.t().contiguous().to(torch.bfloat16)
            dwb = L.lsp_compress_dense_workspace_bytes(m, n, r)
            dws = torch.empty(dwb, dtype=torch.uint8, device=dev)
            S_dense = torch.empty(r, r, device=dev, dtype=torch.float32)
            t_own = timed(lambda G: L.lsp_compress_dense(G, Pdt, Qdt, m, n, r, S_dense, code, dws, dwb, stream), Gs)
            flop = 2.0 * m * n * r + 2.0 * m * r * r
            ref = torch.matmul(Pd.t().double(), torch.matmul(Gs[-1].double(), Qd.double()))   # fp64, fp32 projector values
            scale = ref.abs().max().item()
            rows.append({"m": m, "n": n, "d": d, "sparse_us": round(t_sparse, 1), "dense_mfma_us": round(t_own, 1),
                         "dense_mfma_TFLOP/s": round(flop / t_own / 1e6, 1), "dense_mfma_frac_of_2500": round(flop / t_own / 1e6 / 2500.0, 4),
                         "dense_vendor_gemm_us": round(t_dense, 1),
                         "sparse_max_err_rel": float(f"{(S_sparse.double() - ref).abs().max().item() / scale:.2e}"),
                         "dense_mfma_max_err_rel": float(f"{(S_dense.double() - ref).abs().max().item() / scale:.2e}"),
                         "dense_vendor_max_err_rel": float(f"{(out['S'].double() - ref).abs().max().item() / scale:.2e}")})
            del plan, ws, Pd, Qd, Pdt, Qdb, Qdt, dws, ref
        del Gs
    return {"ablation": "dense projectors (bf16; lsp_compress_dense on the matrix cores, and the vendor GEMM) against the sparse "
                        "compress path, r = 512, bf16 G, one call, one stream, G from HBM", "unit": "us per call",
            "roofline_dense": {"bound": "mfma", "peak": 2500.0, "unit": "TFLOP/s", "flop": "2 m n r + 2 m r^2"}, "rows": rows}


def cpu_baseline(syn, r, d):
    """The oracle, as it stands, on a bounded sample: the fourteen matrices of two layers."""
    import oracle
    cores = len(os.sched_getaffinity(0))
    cores = max(1, min(cores, int(os.environ.get("OMP_NUM_THREADS", cores))))
    total_bytes, total_s = 0, 0.0
    names = []
    for layer, which in [(l, w) for l in (31, 30) for w in range(7)]:     # backward order
        pb = syn.config4_matrix(layer, which)
        t = time.time()
        S = oracle.compress(pb.G, pb.dtype, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, pb.r, threads=cores)
        oracle.decompress_apply(pb.W, pb.dtype, pb.S_in, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, threads=cores)
        total_s += time.time() - t
        total_bytes += pb.compress_bytes + pb.decompress_bytes
        if layer == 31:
            names.append(f"{pb.m}x{pb.n}")
        del S
    # the oracle of the estimation-bias row beyond the step, one 4096 x 4096 matrix (single-threaded as it stands)
    pb = syn.config4_matrix(31, 3)
    t = time.time()
    oracle.estimation_bias(pb.G, pb.dtype, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, pb.r)
    bias_s = time.time() - t
    t = time.time()
    oracle.bias_gradient(pb.G, pb.dtype, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, pb.r)
    grad_s = time.time() - t
    next_rows = {"estimation_bias_s_per_call": round(bias_s, 2), "fitting_gradient_s_per_call": round(grad_s, 2),
                 "sample": "one 4096x4096 bf16 matrix, r=512, d=8, one host thread"}
    return {"value": round(total_bytes / total_s / 1e9, 3), "unit": "GB/s", "cores": cores, "kind": "oracle", "next_rows": next_rows,
            "sample": "compress + decompress-apply of the 14 matrices of two layers (each: " + ", ".join(names) +
                      f"), 1/16 of a step, bf16, r={r}, d={d}; fp64 plain loops, rows split over threads",
            "seconds": round(total_s, 2)}


if __name__ == "__main__":
    main()
