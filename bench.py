#!/usr/bin/env python3
"""Benchmark of the RainFusion hot path on one MI355X.

A step is one pass of the whole path over one synthetic attention layer: ARM classifies
every head from first-frame samples (Alg. 1), then the block-sparse attention runs with the
classes the ARM left on the device (Eq. 1-5).  Inputs are resident in HBM before timing.
Besides the timed steps the script measures, with events on the launch stream, the attention
kernel alone (ARM-chosen classes, the one-third-per-pattern split, and the same kernel run
dense for the speedup figure) and the ARM alone, and times the CPU oracle on a bounded
sample of the same workload.  One JSON line is printed.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA

# HBM-side bytes of one attention launch of the timed step (ARM-chosen classes).  NOT observed by
# this script: copied from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs summarised in
# profiles/attn_kernel_hunyuan720p.md (counter values in KiB, FETCH_SIZE scaled x2.0 and WRITE_SIZE
# x1.0, what the same counters read for a 1 GiB device copy).  Only known for the workload / block
# it was profiled on; the bench line says where the figure comes from.
PROFILED_TRAFFIC_BYTES = {("hunyuan720p", 384): (2.0 * 7.9694e6 + 1.0 * 8.3882e5) * 1024,
                          ("hunyuan720p", 256): (2.0 * 9.5379e6 + 1.0 * 7.5577e5) * 1024}


def kept_pairs(cls, w, bw_s=0.25, bw_t=0.25, tau=2):
    """Token pairs (query, key) one head keeps under a pattern: bookkeeping for FLOP counts."""
    N, Nv, HW, T, tl = w.N, w.Nv, w.HW, w.T, w.text_len
    if cls == 3:
        return N * N

    def band(n, r):
        r = min(r, n - 1)
        return n * (2 * r + 1) - r * (r + 1)

    if cls == 0:
        vv = band(T, math.floor(float(bw_s) * T)) * HW * HW
    elif cls == 1:
        vv = band(HW, math.floor(float(bw_t) * HW)) * T * T
    else:
        per_frame = sum(1 for y in range(w.H) for x in range(w.W) if (y - x) % tau == 0)
        vv = Nv * per_frame * T
    return vv + tl * N + Nv * tl  # text rows see everything, video rows see every text key


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="hunyuan720p")
    ap.add_argument("--block", type=int, default=0, help="query rows per block (64|128|256|384); 0 = the workload's")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--wide-rows", action="store_true",
                    help="run the attention with RF_FLAG_WIDE_ROWS (64 query rows per wavefront; head_dim 128, block 256)")
    ap.add_argument("--fixed-order", action="store_true",
                    help="run the attention with RF_FLAG_FIXED_ORDER (bitwise reproducible tile order)")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the step: time the bandwidth / stride settings of the paper's sensitivity "
                         "table (w = 0.25/0.18/0.13, tau = 2/3/4) against the dense run; prints one JSON line")
    ap.add_argument("--plus", action="store_true",
                    help="instead of the step: time RainFusion+ (per-head bandwidth from 0.5/0.25/0.125) on the "
                         "planted workload, whose heads the ARM can tell apart; prints one JSON line")
    ap.add_argument("--configs", action="store_true",
                    help="instead of the step: the other named configurations, each against the same kernel run dense: "
                         "the CogVideoX-shaped layer with round-robin classes and with ARM-chosen classes (equal-interval "
                         "sampling), the Open-Sora-Plan-shaped layer at blocks 128 and 256, the planted layer at blocks "
                         "64 and 128 with ARM-chosen classes; prints one JSON line")
    ap.add_argument("--only", default="", help="profiling aid: run just 'step', 'arm', 'thirds', 'dense', every head 'spatial' / 'temporal' / 'textural', or 'copy' (a 1 GiB device copy)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no sharding, no collectives); use --gpus 1")

    import torch

    import paper_2505_21036_amd as rf
    import rf_inputs as inp

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    if args.configs:
        args.workload = "tiny"  # --configs brings its own workloads; keep the common set-up below small
    w = inp.WORKLOADS[args.workload]
    block = args.block or w.block
    rl = rf.rf_layout(w.T, w.H, w.W, w.text_len)
    Q, K, V = inp.full_qkv(w, dev)
    O = torch.empty_like(Q)
    hc = torch.empty(w.B, w.nH, dtype=torch.int32, device=dev)
    rec = torch.empty(w.B, w.nH, 2, dtype=torch.float32, device=dev)
    ws = torch.empty(max(rf.rf_arm_workspace_bytes(w.B, w.nH, rl), 4), dtype=torch.uint8, device=dev)
    ws_attn = torch.empty(rf.rf_attention_workspace_bytes(w.B, w.nH, w.D, rl), dtype=torch.uint8, device=dev)
    thirds = inp.thirds_classes(w).to(dev)
    dense = torch.full((w.B, w.nH), rf.RF_DENSE, dtype=torch.int32, device=dev)

    def arm():
        rf.rf_arm_classify(Q, K, rl, None, rf.RF_SAMPLE_FIRST_FRAME, 0.9, hc, rec, ws)

    attn_flags = (rf.RF_FLAG_FIXED_ORDER if args.fixed_order else 0) | (rf.RF_FLAG_WIDE_ROWS if args.wide_rows else 0)
    attn_params = rf.rf_params(0.25, 0.25, 2, 0, attn_flags) if attn_flags else None

    def attn(classes):
        rf.rf_sparse_attention(Q, K, V, classes, rl, attn_params, block, O, ws_attn)

    def step():
        arm()
        attn(hc)

    def event_ms(fn, reps):
        """Average duration of fn's launches, events recorded on the stream the kernels run on."""
        pairs = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            pairs.append((a, b))
        torch.cuda.synchronize()
        return sum(a.elapsed_time(b) for a, b in pairs) / reps

    if args.sweep:
        attn(dense)
        ms_dense = event_ms(lambda: attn(dense), 2)
        rows = []
        for bw, tau, paper in ((0.25, 2, 1.85), (0.18, 3, 2.50), (0.13, 4, 3.00)):
            prm = rf.rf_params(bw, bw, tau, 0, 0)
            ws_s = torch.empty(rf.rf_attention_workspace_bytes(w.B, w.nH, w.D, rl, prm), dtype=torch.uint8, device=dev)
            row = {"bandwidth": bw, "tex_stride": tau, "paper_speedup_with_10pct_dense_steps": paper}
            for name, classes in (("spatial", torch.zeros_like(dense)), ("temporal", torch.ones_like(dense)),
                                  ("textural", torch.full_like(dense, 2)), ("thirds", thirds)):
                fn = lambda: rf.rf_sparse_attention(Q, K, V, classes, rl, prm, block, O, ws_s)
                fn()
                ms = event_ms(fn, 2)
                kept = sum(kept_pairs(c, w, bw, bw, tau) for c in classes.cpu().flatten().tolist()) / (w.B * w.nH * w.N * w.N)
                row[name] = {"ms": round(ms, 3), "speedup_vs_dense": round(ms_dense / ms, 3),
                             "kept_fraction": round(kept, 4), "flop_count_speedup": round(1 / kept, 3),
                             "speedup_if_10pct_steps_dense": round(1 / (0.1 + 0.9 * ms / ms_dense), 3)}
            rows.append(row)
        print(json.dumps({"sweep": rows, "dense_ms": round(ms_dense, 3), "workload": w.name, "block": block}))
        return

    if args.plus:
        wp = inp.WORKLOADS["planted"]
        rlp = rf.rf_layout(wp.T, wp.H, wp.W, wp.text_len)
        Qp, Kp, Vp = inp.full_qkv(wp, dev)
        bws = [0.5, 0.25, 0.125]
        hc_p, hbw_p, _ = rf.rf_arm_classify_plus(Qp, Kp, rlp, None, rf.RF_SAMPLE_FIRST_FRAME, 0.9, bws)
        hc_b, _ = rf.rf_arm_classify(Qp, Kp, rlp, None, rf.RF_SAMPLE_FIRST_FRAME, 0.9)
        dense_p = torch.full_like(hc_p, rf.RF_DENSE)
        Op = torch.empty_like(Qp)
        runs = {"arm_plus": lambda: rf.rf_arm_classify_plus(Qp, Kp, rlp, None, rf.RF_SAMPLE_FIRST_FRAME, 0.9, bws),
                "arm_base": lambda: rf.rf_arm_classify(Qp, Kp, rlp, None, rf.RF_SAMPLE_FIRST_FRAME, 0.9),
                "attention_plus": lambda: rf.rf_sparse_attention_plus(Qp, Kp, Vp, hc_p, hbw_p, bws, rlp, None, wp.block, Op),
                "attention_base": lambda: rf.rf_sparse_attention(Qp, Kp, Vp, hc_b, rlp, None, wp.block, Op),
                "attention_dense": lambda: rf.rf_sparse_attention(Qp, Kp, Vp, dense_p, rlp, None, wp.block, Op)}
        res = {}
        for name, fn in runs.items():
            fn()
            res[name + "_ms"] = round(event_ms(fn, 5), 4)
        hist = {}
        for c, b in zip(hc_p.cpu().flatten().tolist(), hbw_p.cpu().flatten().tolist()):
            key = "%s@%s" % (("spatial", "temporal", "textural", "dense")[c], bws[b] if b >= 0 else "-")
            hist[key] = hist.get(key, 0) + 1
        res.update({"workload": wp.name, "block": wp.block, "candidates": bws, "chosen": hist,
                    "speedup_plus_vs_dense": round(res["attention_dense_ms"] / res["attention_plus_ms"], 3),
                    "speedup_base_vs_dense": round(res["attention_dense_ms"] / res["attention_base_ms"], 3)})
        print(json.dumps({"plus": res}))
        return

    if args.configs:
        del Q, K, V, O, ws_attn
        torch.cuda.empty_cache()
        rows = []

        def time_config(name, blocks, arm_mode=None, forced=None):
            wc = inp.WORKLOADS[name]
            rlc = rf.rf_layout(wc.T, wc.H, wc.W, wc.text_len)
            Qc, Kc, Vc = inp.full_qkv(wc, dev)
            Oc = torch.empty_like(Qc)
            wsc = torch.empty(rf.rf_attention_workspace_bytes(wc.B, wc.nH, wc.D, rlc), dtype=torch.uint8, device=dev)
            densec = torch.full((wc.B, wc.nH), rf.RF_DENSE, dtype=torch.int32, device=dev)
            row = {"workload": "%s: B%d nH%d D%d, %d frames x %dx%d + %d text = %d tokens" % (
                wc.name, wc.B, wc.nH, wc.D, wc.T, wc.H, wc.W, wc.text_len, wc.N)}
            if arm_mode is not None:
                hcc, _ = rf.rf_arm_classify(Qc, Kc, rlc, None, arm_mode, 0.9)
                row["classes"] = "chosen by the ARM (%s sampling)" % ("first-frame", "equal-interval")[arm_mode]
                armf = lambda: rf.rf_arm_classify(Qc, Kc, rlc, None, arm_mode, 0.9)
                armf()
                row["arm_ms"] = round(event_ms(armf, 5), 4)
            else:
                hcc = forced(wc).to(dev)
                row["classes"] = forced.__name__
            ch = hcc.cpu().flatten().tolist()
            row["class_histogram"] = {"spatial": ch.count(0), "temporal": ch.count(1), "textural": ch.count(2), "dense": ch.count(3)}
            kept = sum(kept_pairs(c, wc) for c in ch) / float(wc.B * wc.nH * wc.N * wc.N)
            row["kept_fraction"] = round(kept, 4)
            for blk in blocks:
                sparse = lambda: rf.rf_sparse_attention(Qc, Kc, Vc, hcc, rlc, None, blk, Oc, wsc)
                densef = lambda: rf.rf_sparse_attention(Qc, Kc, Vc, densec, rlc, None, blk, Oc, wsc)
                sparse()
                ms = event_ms(sparse, 5)
                densef()
                msd = event_ms(densef, 3)
                row["block_%d" % blk] = {"sparse_ms": round(ms, 4), "dense_ms": round(msd, 4), "speedup_vs_dense": round(msd / ms, 3),
                                         "flop_count_speedup": round(1 / kept, 3),
                                         "tflops_useful": round(kept * wc.dense_flops() / ms / 1e9, 1),
                                         "tflops_dense": round(wc.dense_flops() / msd / 1e9, 1),
                                         "mfma_frac_dense": round(wc.dense_flops() / msd / 1e9 / PEAK_BF16_TFLOPS, 4)}
                if "arm_ms" in row:
                    row["block_%d" % blk]["arm_pct_of_sparse_attention"] = round(100 * row["arm_ms"] / ms, 3)
            rows.append(row)

        time_config("cogvideox", (128, 256), forced=inp.round_robin_classes)
        time_config("cogvideox", (128, 256), arm_mode=rf.RF_SAMPLE_EQUAL_INTERVAL)
        time_config("osp720p", (128, 256, 384), forced=inp.thirds_classes)
        time_config("planted", (64, 128), arm_mode=rf.RF_SAMPLE_FIRST_FRAME)
        print(json.dumps({"configs": rows}))
        return

    if args.only:
        one = {n: torch.full((w.B, w.nH), c, dtype=torch.int32, device=dev)
               for n, c in (("spatial", rf.RF_SPATIAL), ("temporal", rf.RF_TEMPORAL), ("textural", rf.RF_TEXTURAL))}
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev) if args.only == "copy" else None
        dst = torch.empty_like(src) if src is not None else None
        fn = {"step": step, "arm": arm, "thirds": lambda: attn(thirds), "dense": lambda: attn(dense),
              "copy": lambda: dst.copy_(src),  # 1 GiB read + 1 GiB written: calibrates FETCH_SIZE / WRITE_SIZE
              "spatial": lambda: attn(one["spatial"]), "temporal": lambda: attn(one["temporal"]),
              "textural": lambda: attn(one["textural"])}[args.only]
        arm()
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        print(json.dumps({"only": args.only, "ms": (time.perf_counter() - t0) * 1e3 / args.steps}))
        return

    # ---- the timed region: K whole steps, attention launches bracketed by stream events
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        arm()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        attn(hc)
        b.record()
        ev.append((a, b))
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) * 1e3 / args.steps
    ms_attn_arm_classes = sum(a.elapsed_time(b) for a, b in ev) / args.steps
    classes_host = hc.cpu().flatten().tolist()
    recalls_host = rec.cpu().reshape(-1, 2).tolist()

    reps = max(2, min(args.steps, 5))
    ms_arm = event_ms(arm, reps)
    attn(thirds)
    ms_thirds = event_ms(lambda: attn(thirds), reps)
    attn(dense)
    ms_dense = event_ms(lambda: attn(dense), max(2, reps // 2))

    # ---- the same step on planted heads of the same shape, where the ARM picks all three patterns
    planted = None
    wp = inp.WORKLOADS.get(w.name + "_planted")
    if wp is not None:
        Qp, Kp, Vp = inp.full_qkv(wp, dev)

        def planted_step():
            rf.rf_arm_classify(Qp, Kp, rl, None, rf.RF_SAMPLE_FIRST_FRAME, 0.9, hc, rec, ws)
            rf.rf_sparse_attention(Qp, Kp, Vp, hc, rl, None, block, O, ws_attn)

        planted_step()
        torch.cuda.synchronize()
        evp = []
        t0 = time.perf_counter()
        for _ in range(reps):
            rf.rf_arm_classify(Qp, Kp, rl, None, rf.RF_SAMPLE_FIRST_FRAME, 0.9, hc, rec, ws)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            rf.rf_sparse_attention(Qp, Kp, Vp, hc, rl, None, block, O, ws_attn)
            b.record()
            evp.append((a, b))
        torch.cuda.synchronize()
        ms_planted_step = (time.perf_counter() - t0) * 1e3 / reps
        ms_planted_attn = sum(a.elapsed_time(b) for a, b in evp) / reps
        pc = hc.cpu().flatten().tolist()
        want = [inp.planted_class(wp, b, h) for b in range(wp.B) for h in range(wp.nH)]
        useful_p = 4.0 * w.D * sum(kept_pairs(c, w) for c in pc)
        planted = {"planted_step_ms": round(ms_planted_step, 4), "planted_attention_ms": round(ms_planted_attn, 4),
                   "planted_arm_classes": {"spatial": pc.count(0), "temporal": pc.count(1), "textural": pc.count(2)},
                   "planted_classes_recovered": pc == want,
                   "planted_useful_flop_fraction": round(useful_p / w.dense_flops(), 4),
                   "planted_tflops_useful": round(useful_p / ms_planted_attn / 1e9, 2),
                   "planted_mfma_frac_useful": round(useful_p / ms_planted_attn / 1e9 / PEAK_BF16_TFLOPS, 4),
                   "planted_speedup_vs_dense": round(ms_dense / ms_planted_attn, 3)}
        del Qp, Kp, Vp
        arm()  # leave the i.i.d. classes in hc again

    # ---- FLOP bookkeeping: 4*D flops per (query, key) pair for QK^T and PV
    per_pair = 4.0 * w.D
    thirds_host = thirds.cpu().flatten().tolist()
    useful_arm = per_pair * sum(kept_pairs(c, w) for c in classes_host)
    useful_thirds = per_pair * sum(kept_pairs(c, w) for c in thirds_host)

    def executed(classes):
        tot = 0
        for c in set(classes):
            # Temporal heads walk the position-major copy (the workspace is always given here)
            vis, _, _ = rf.plan_block_counts(rl, None, block, rf.RF_LIST_TEMPORAL_POSITION_MAJOR if c == 1 else c)
            tot += vis * classes.count(c)
        return per_pair * block * rf.RF_KEY_TILE * tot

    exec_arm, exec_thirds = executed(classes_host), executed(thirds_host)
    dense_flops = w.dense_flops()
    arm_flops = 2.0 * w.D * 2 * w.HW * w.HW * w.nH * w.B  # two passes of ~HW x HW scores per head

    out = {
        "metric": "sparse_attn_ms_per_layer",
        "value": round(ms_step, 4),
        "unit": "ms",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": "%s: B%d nH%d D%d, %d frames x %dx%d + %d text tokens = %d tokens, i.i.d. N(0,1)/sqrt(D) bf16; "
                        "step = ARM (first-frame sampling, threshold 0.9) + block-sparse attention with the classes "
                        "the ARM chose" % (w.name, w.B, w.nH, w.D, w.T, w.H, w.W, w.text_len, w.N),
            "block": block,
            "bandwidth": 0.25,
            "tex_stride": 2,
            "arm_classes": {"spatial": classes_host.count(0), "temporal": classes_host.count(1),
                            "textural": classes_host.count(2)},
        },
        "roofline": {
            "kernel": "attn_kernel<%d,%d> (ARM-chosen classes)" % (w.D, block // 32),
            "bound": "mfma",
            "achieved": round(useful_arm / ms_attn_arm_classes / 1e9, 2),
            "peak": PEAK_BF16_TFLOPS,
            "unit": "TFLOP/s",
            "frac": round(useful_arm / ms_attn_arm_classes / 1e9 / PEAK_BF16_TFLOPS, 4),
            "traffic": PROFILED_TRAFFIC_BYTES.get((w.name, block)),
            "traffic_source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE run recorded in profiles/attn_kernel_hunyuan720p.md; "
                              "not observed by this run",
            "traffic_gbps_at_this_runs_time": (round(PROFILED_TRAFFIC_BYTES[(w.name, block)] / ms_attn_arm_classes / 1e6, 1)
                                               if (w.name, block) in PROFILED_TRAFFIC_BYTES else None),
            "algorithmic_bytes": 8.0 * w.N * w.D * w.nH * w.B,
            "algorithmic_gbps": round(8.0 * w.N * w.D * w.nH * w.B / ms_attn_arm_classes / 1e6, 1),
        },
        "detail": {
            "attention_ms_arm_classes": round(ms_attn_arm_classes, 4),
            "attention_ms_thirds_split": round(ms_thirds, 4),
            "attention_ms_dense_same_kernel": round(ms_dense, 4),
            "speedup_vs_dense_arm_classes": round(ms_dense / ms_attn_arm_classes, 3),
            "speedup_vs_dense_thirds_split": round(ms_dense / ms_thirds, 3),
            "arm_ms": round(ms_arm, 4),
            "arm_pct_of_sparse_attention": round(100.0 * ms_arm / ms_attn_arm_classes, 3),
            "arm_tflops": round(arm_flops / ms_arm / 1e9, 2),
            "tflops_useful_arm_classes": round(useful_arm / ms_attn_arm_classes / 1e9, 2),
            "tflops_executed_arm_classes": round(exec_arm / ms_attn_arm_classes / 1e9, 2),
            "tflops_useful_thirds": round(useful_thirds / ms_thirds / 1e9, 2),
            "tflops_executed_thirds": round(exec_thirds / ms_thirds / 1e9, 2),
            "tflops_dense": round(dense_flops / ms_dense / 1e9, 2),
            "dense_equivalent_tflops_thirds": round(dense_flops / ms_thirds / 1e9, 2),
            "kept_fraction_thirds": round(useful_thirds / dense_flops, 4),
            "executed_fraction_thirds": round(exec_thirds / dense_flops, 4),
            "mfma_frac_dense": round(dense_flops / ms_dense / 1e9 / PEAK_BF16_TFLOPS, 4),
            "recalls_head0": [round(x, 4) for x in recalls_host[0]],
            "paper_context": "paper reports 1.84-1.91x attention speedup (hardware not stated), ARM ~0.2 %",
        },
    }
    if planted:
        out["detail"].update(planted)

    if not args.no_cpu_baseline:
        import numpy as np

        import oracle as orc
        ol = orc.Layout(w.T, w.H, w.W, w.text_len)
        q, k, v = (t.float().numpy() for t in inp.head_qkv(w, 0, 0))
        nthreads = orc.num_threads()
        rows = np.array(inp.sample_rows(w, 1536 * nthreads))  # ~10-30 s of oracle time
        cls0 = classes_host[0]
        orc.attention_rows(q, k, v, cls0, ol, orc.Params(), rows[:nthreads])  # warm the library / threads
        t0 = time.perf_counter()
        orc.attention_rows(q, k, v, cls0, ol, orc.Params(), rows)
        t_rows = time.perf_counter() - t0
        t0 = time.perf_counter()
        orc.arm_classify(q, k, ol, orc.Params(), orc.SAMPLE_FIRST_FRAME, 0.9)
        t_arm = time.perf_counter() - t0
        layer_ms = (t_rows / len(rows) * w.N + t_arm) * w.nH * w.B * 1e3
        out["cpu_baseline"] = {
            "value": round(layer_ms, 1),
            "unit": "ms",
            "cores": nthreads,
            "kind": "oracle",
            "sample": "fp64 oracle on head (0,0): %d complete query rows of class %d in %.2f s plus the full ARM of "
                      "that head in %.2f s, scaled by N*nH*B/rows to one layer" % (len(rows), cls0, t_rows, t_arm),
        }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
