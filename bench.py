#!/usr/bin/env python3
"""Benchmark of the QuantuneV2 sensitivity pass on one MI355X.

One step = one pass of the whole hot path over the layer table: calibrate
(min/max, statistics, scale, zero-point) -> fake-quantize (int8 codes, error
energies) -> pair metrics (fp32-run vs quantized-run activations) -> fold the
segment records to one per tensor on the device and copy those few KB to the
host -> finalize (MSE, SQNR, mean, var) -> SQNR delta and ranking.  Inputs are synthetic, seeded, and resident in HBM before
the timed region starts.

Workload at N=1: ResNet-50 v1 shapes, batch 256, 224x224 (54 weights,
per-output-channel symmetric; 54 activations with their quantized-run partners,
per-tensor asymmetric).

Prints ONE JSON line.  `value` is algorithmic bytes per pass / time per pass with
the fixed per-call numerators: 4 B/element for calibrate, 5 for fake-quant (4 read
+ 1 code written), 8 for the pair metrics, i.e. 9 B per weight element and 17 B
per activation element.  The default pass is the single call
qv2_calibrate_fakequant_pair_metrics, which computes the same results while moving
13 B per activation element (fake-quant and pair comparison share one visit of x)
and 5 B per element of the per-channel weights (read once, staged in LDS); the
JSON also carries `hbm_GBps` (bytes the pass actually has to move / time) and the
timing of the pass made of the three separate calls.
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

HBM_PEAK_GBPS = 8000.0   # MI355X published HBM3E bandwidth
ROCPROF_NAMES = {"k_statspair_stream": "k_stats_stream<512, 8, true, false>",
                 "k_quantpair_stream": "k_quant_stream<256, 2, true, false, true, false>", "k_pair_stream": "k_pair_stream<512, 4>"}

# HBM bytes per launch of the dominant kernel on the resnet50 b256 workload from rocprofv3
# --pmc (FETCH_SIZE and WRITE_SIZE runs, each scaled by a copy kernel of known size); see
# profiles/sensitivity_pass_resnet50_b256.txt.
TRAFFIC_BYTES = {"k_statspair_stream": 21_697_364_277, "k_pair_stream": 21_697_202_899,
                 "k_quantpair_stream": 24_627_581_264}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="resnet50", choices=["resnet50", "resnet18", "vgg16", "mobilenetv2"])
    ap.add_argument("--batch", type=int, default=None, help="override the workload's batch (smaller = not the headline config)")
    ap.add_argument("--fused", action="store_true", help="BN-folded weight variant of resnet50")
    ap.add_argument("--mode", default="single", choices=["single", "fused", "calls"],
                    help="single: the one call that calibrates, fake-quantizes and compares with the "
                         "quantized run (default); fused: calibrate + fused fake-quant/pair call; "
                         "calls: calibrate, fake-quant and pair as three calls")
    ap.add_argument("--single-mode", action="store_true", help="do not also time the other mode")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--checksums", action="store_true",
                    help="print one checksum line per input tensor to stderr (the JSON line always carries "
                         "their combination as config.inputs_checksum)")
    ap.add_argument("--cpu-sample-elems", type=int, default=2_000_000_000)
    ap.add_argument("--no-cold", dest="cold", action="store_false",
                    help="skip the second timing in which every step follows a 1 GiB fill that evicts the "
                         "256 MB Infinity Cache (reported as `cold`; it matters only for sets that are not "
                         "far larger than that cache)")
    ap.add_argument("--cold", dest="cold", action="store_true", help="(default) see --no-cold")
    ap.set_defaults(cold=True)
    ap.add_argument("--no-single-tensor-extra", action="store_true",
                    help="skip the 1600 tiny fake-quant calls of extras.fakequant_single_tensor_us (profiling runs)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="after the timed region also run 3 plain 1 GiB device copies (a kernel of known "
                         "traffic, used to scale rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    return ap.parse_args()


def build_workload(args, dev):
    import torch
    from paper_2501_07161_amd import binding as qb
    from paper_2501_07161_amd import synth

    defaults = {"resnet50": 256, "resnet18": 32, "vgg16": 16, "mobilenetv2": 64}
    batch = args.batch or defaults[args.workload]
    if args.workload == "resnet50":
        specs = synth.config_resnet50(batch, fused=args.fused)
    elif args.workload == "vgg16":
        specs = synth.config_vgg16(batch, per_channel=True)
    else:
        specs = synth.CONFIGS[args.workload](batch)
    xs = [synth.materialize(s, dev) for s in specs]
    codes = [torch.empty(x.numel(), dtype=torch.int8, device=dev) for x in xs]

    # quantized-run partners: dequant(quant(ref)) + N(0, (0.01 std(ref))^2).  Built here with
    # the library's own calibrate / fake-quant (untimed set-up) and plain torch arithmetic.
    rows0 = [qb.TensorArg(x=x, numel=x.numel(), scheme=s.scheme, channels=s.channels, codes=c,
                          kind=s.kind, layer=s.layer) for x, s, c in zip(xs, specs, codes)]
    plan0 = qb.qv2_plan_create(rows0)
    buf0 = qb.Buffers(plan0, dev)
    qb.qv2_calibrate(plan0, buf0.params, buf0.sums, buf0.workspace)
    qb.qv2_fakequant_metrics(plan0, buf0.params, buf0.sums, buf0.workspace)
    torch.cuda.synchronize()
    params, _, _ = buf0.host()
    qruns = []
    for t, (s, x, c) in enumerate(zip(specs, xs, codes)):
        if not s.has_pair:
            qruns.append(None)
            continue
        p = params[plan0.segment_begin[t]]
        q = c.view(x.shape).to(torch.float32).sub_(float(p["zp"])).mul_(float(p["scale"]))
        q.add_(synth.unit_noise(s, dev), alpha=0.01 * float(x.std(unbiased=False)))
        qruns.append(q)
    plan0.close()
    del buf0
    rows = [qb.TensorArg(x=x, numel=x.numel(), scheme=s.scheme, channels=s.channels, qrun=q, codes=c,
                         kind=s.kind, layer=s.layer) for x, s, q, c in zip(xs, specs, qruns, codes)]
    return specs, xs, qruns, codes, rows, batch


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build runs on ONE GPU; --gpus {args.gpus} is not supported "
              "(no collectives or sharding are part of it).", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2501_07161_amd import binding as qb
    from paper_2501_07161_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    qb.lib()                                  # raises if libqv2.so has not been built
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    specs, xs, qruns, codes, rows, batch = build_workload(args, dev)
    plan = qb.qv2_plan_create(rows)
    buf = qb.Buffers(plan, dev)
    n_layers = max(s.layer for s in specs) + 1
    n_w = sum(s.numel for s in specs if s.kind == synth.WEIGHT)
    n_a = sum(s.numel for s in specs if s.kind == synth.ACTIVATION)
    n_pair = sum(s.numel for s, q in zip(specs, qruns) if q is not None)
    n_all = n_w + n_a
    n_rowgroup = sum(s.numel for s in specs if s.scheme == synth.SYM_CHANNEL and s.numel // s.channels <= 8192)
    bytes_cal, bytes_fq, bytes_pair = 4 * n_all, 5 * n_all, 8 * n_pair
    bytes_pass = bytes_cal + bytes_fq + bytes_pair

    # pinned host mirrors of the small result records
    # per-tensor records and pair sums share one device buffer, so one copy brings both back
    n_ts = plan.num_tensors * qb.TENSOR_SUMS.itemsize
    d_out = torch.zeros(n_ts + plan.num_tensors * qb.PAIR_SUMS.itemsize, dtype=torch.uint8, device=dev)
    d_tsums, d_pair = d_out[:n_ts], d_out[n_ts:]
    h_out = torch.empty(d_out.shape, dtype=torch.uint8, pin_memory=True)
    h_tsums_np = h_out[:n_ts].numpy().view(qb.TENSOR_SUMS)
    h_pair_np = h_out[n_ts:].numpy().view(qb.PAIR_SUMS)
    buf.pair = d_pair
    last = {}

    pout = qb.PassOutputs(plan, n_layers, dev)

    def step(mode, events=None):
        if events:
            events[0].record()
        if mode == "single":
            # steps 1-4 in ONE native call: device pass, per-tensor fold, one copy of a few KB,
            # Eq. 6-7, Eq. 16 and Algorithm 2; it returns with the list made
            order, score = qb.qv2_sensitivity_pass(plan, buf.params, buf.sums, pout, buf.workspace)
            if events:
                events[1].record()
                events[3].record()
                kernel_log.append(qb.qv2_plan_kernels_ms(plan).copy())
            last.update(order=order, score=score, met=pout.metrics, pmse=pout.pair_mse, psqnr=pout.pair_sqnr_db)
            return
        else:
            qb.qv2_calibrate(plan, buf.params, buf.sums, buf.workspace)
        if events:
            events[1].record()
        if mode == "fused":
            qb.qv2_fakequant_pair_metrics(plan, buf.params, buf.sums, buf.pair, buf.workspace)
        else:
            qb.qv2_fakequant_metrics(plan, buf.params, buf.sums, buf.workspace)
            if events:
                events[2].record()
            qb.qv2_pair_metrics(plan, buf.pair, buf.workspace)
        if events:
            events[3].record()
        # per-tensor records are folded on the device: a few KB go to the host, not every segment
        qb.qv2_tensor_sums_fold(plan, buf.params, buf.sums, d_tsums)
        h_out.copy_(d_out, non_blocking=True)
        torch.cuda.current_stream().synchronize()
        if events:       # per-kernel durations from the library's HIP events on the same stream
            kernel_log.append(qb.qv2_plan_kernels_ms(plan).copy())
        ts, ps = h_tsums_np, h_pair_np
        met = qb.qv2_finalize_tensors(ts)                    # per tensor: MSE, SQNR, mean, var, absmax
        pmse, psqnr = qb.qv2_pair_finalize(ps)               # per activation pair: MSE, SQNR
        order, score = qb.qv2_rank_tensors(plan, ts, ps, n_layers)   # per-layer series, Eq. 16, Algorithm 2
        last.update(order=order, score=score, met=met, pmse=pmse, psqnr=psqnr)

    kernel_ms, kernel_log = {}, []
    qb.qv2_plan_set_timing(plan, True)

    def timed(mode):
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
        kernel_ms.clear()
        names = {"single": ["k_statspair_stream", "k_quant_stream", "k_single_read_rows"],
                 "fused": ["k_stats_stream", "k_stats_rows", "k_quantpair_stream", "k_quantpair_rows"],
                 "calls": ["k_stats_stream", "k_stats_rows", "k_quant_stream", "k_quant_rows", "k_pair_stream"]}[mode]
        kernel_log.clear()
        for _ in range(args.warmup):
            step(mode)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        marks = [t0]
        for k in range(args.steps):
            step(mode, ev[k])          # ends with the ranking on the host, so each step is complete here
            marks.append(time.perf_counter())
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        per_step = np.diff(marks) * 1e3
        kernel_ms.update({n: [row[qb.KERNEL_IDS[n]] for row in kernel_log] for n in names})
        r = {"ms_per_step": dt / args.steps * 1e3, "ms_median": float(np.median(per_step)),
             "ms_min": float(np.min(per_step)), "order": last["order"].tolist(),
             "kernels_ms": {n: round(float(np.mean(v)), 4) for n, v in kernel_ms.items()},
             "ms_cal": float(np.mean([e[0].elapsed_time(e[1]) for e in ev]))}
        if mode == "single":
            r["ms_single"] = r.pop("ms_cal")
        elif mode == "fused":
            r["ms_fqpair"] = float(np.mean([e[1].elapsed_time(e[3]) for e in ev]))
        else:
            r["ms_fq"] = float(np.mean([e[1].elapsed_time(e[2]) for e in ev]))
            r["ms_pair"] = float(np.mean([e[2].elapsed_time(e[3]) for e in ev]))
        return r

    main_r = timed(args.mode)
    cold_ms = None
    if args.cold:
        scratch = torch.empty(1 << 28, dtype=torch.float32, device=dev)
        ts = []
        for _ in range(args.steps):
            scratch.fill_(1.0)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            step(args.mode)
            torch.cuda.synchronize()
            ts.append(time.perf_counter() - t0)
        cold_ms = float(np.mean(ts)) * 1e3
        del scratch
    other_mode = "fused" if args.mode == "calls" else "calls"
    other = None if args.single_mode else timed(other_mode)

    # optional metrics outside the headline pass (the paper's other candidate local metrics)
    extras = {}
    if not args.single_mode:
        nb = 2048
        hx = torch.zeros(plan.num_tensors * nb, dtype=torch.int64, device=dev)
        hq = torch.zeros(plan.num_tensors * nb, dtype=torch.int64, device=dev)
        hws = torch.zeros(qb.qv2_histogram_workspace_bytes(plan, nb), dtype=torch.uint8, device=dev)
        sxh = torch.zeros(plan.num_segments, dtype=torch.float64, device=dev)
        pxq = torch.zeros(plan.num_tensors, dtype=torch.float64, device=dev)
        t_h, t_c, t_s = [], [], []
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for it in range(5):
            qb.qv2_histogram(plan, buf.params, nb, hx, hq, hws)
            qb.qv2_fakequant_pair_metrics_cos(plan, buf.params, buf.sums, buf.pair, sxh, pxq, buf.workspace)
            torch.cuda.synchronize()
            if it >= 1:
                t_h.append(qb.qv2_plan_kernel_ms(plan, "k_hist"))
                t_c.append(qb.qv2_plan_kernel_ms(plan, "k_quantpair_stream"))
            e0.record()
            qb.qv2_calibrate_fakequant_pair_metrics_cos(plan, buf.params, buf.sums, buf.pair, sxh, pxq,
                                                        buf.workspace)
            e1.record()
            torch.cuda.synchronize()
            if it >= 1:
                t_s.append(e0.elapsed_time(e1))
        # the same single call for a caller that wants the metrics only (no code buffers): the
        # quantize sweep then stores nothing and runs over long read-only tiles
        rows_m = [qb.TensorArg(x=r.x, numel=r.numel, scheme=r.scheme, channels=r.channels, qrun=r.qrun,
                               kind=r.kind, layer=r.layer) for r in rows]
        plan_m = qb.qv2_plan_create(rows_m)
        buf_m = qb.Buffers(plan_m, dev)
        t_m = []
        for it in range(5):
            e0.record()
            qb.qv2_calibrate_fakequant_pair_metrics(plan_m, buf_m.params, buf_m.sums, buf_m.pair, buf_m.workspace)
            e1.record()
            torch.cuda.synchronize()
            if it >= 1:
                t_m.append(e0.elapsed_time(e1))
        plan_m.close()
        del buf_m
        hist_bytes = 4 * n_all + 4 * n_pair
        extras = {"histogram_2048_bins": {"kernel_ms": round(float(np.mean(t_h)), 4),
                                          "GBps": round(hist_bytes / np.mean(t_h) / 1e6, 1)},
                  "fused_quantize_with_cosine": {"kernel_ms": round(float(np.mean(t_c)), 4)},
                  "single_call_with_cosine": {"call_ms": round(float(np.mean(t_s)), 4)},
                  "single_call_metrics_only": {"call_ms": round(float(np.mean(t_m)), 4),
                                               "moved_bytes": 8 * n_all + 4 * n_pair - 4 * n_rowgroup,
                                               "GBps": round((8 * n_all + 4 * n_pair - 4 * n_rowgroup)
                                                             / np.mean(t_m) / 1e6, 1)}}
        del hx, hq, hws
        # quantize + dequantize + error of single batch-1 activations (the shapes of the paper's
        # Q-DQ overhead table, Sec. 7; its 341-1518 us per tensor are from other hardware: context)
        qdq = {}
        shapes = () if args.no_single_tensor_extra else ((1, 256, 56, 56), (1, 512, 28, 28), (1, 1024, 14, 14),
                                                         (1, 2048, 7, 7))
        for shp in shapes:
            t1 = torch.randn(shp, device=dev).clamp_(min=0)
            c1 = torch.empty(t1.numel(), dtype=torch.int8, device=dev)
            p1 = qb.qv2_plan_create([qb.TensorArg(x=t1, numel=t1.numel(), codes=c1)])
            b1 = qb.Buffers(p1, dev)
            qb.qv2_calibrate(p1, b1.params, b1.sums, b1.workspace)            # cached parameters
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            for rep in range(2):
                e0.record()
                for _ in range(200):
                    qb.qv2_fakequant_metrics(p1, b1.params, b1.sums, b1.workspace)
                e1.record()
                torch.cuda.synchronize()
            qdq["x".join(map(str, shp))] = round(e0.elapsed_time(e1) / 200 * 1e3, 2)
            p1.close()
        if qdq:
            extras["fakequant_single_tensor_us"] = qdq

    if args.copy_probe:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    ms_per_step = main_r["ms_per_step"]
    value = bytes_pass / (ms_per_step * 1e-3) / 1e9
    # bytes the executed pass has to move: the fused call reads x once for steps a3 + a4
    bytes_fqpair = 5 * n_all + 4 * n_pair
    # ... and the single call reads the tensors made of short channels once for a1 + a3 too
    bytes_single = bytes_cal + bytes_fqpair - 4 * n_rowgroup
    moved_of = {"single": bytes_single, "fused": bytes_cal + bytes_fqpair, "calls": bytes_cal + bytes_fq + bytes_pair}
    moved = moved_of[args.mode]
    headline = args.workload == "resnet50" and batch == 256 and not args.fused

    def calls_of(r):
        if "ms_single" in r:       # one host call that also waits, finalizes and ranks
            return {"sensitivity_pass": {"ms": round(r["ms_single"], 4), "moved_bytes": bytes_single,
                                         "GBps": round(bytes_single / r["ms_single"] / 1e6, 1)}}
        c = {"calibrate": {"ms": round(r["ms_cal"], 4), "GBps": round(bytes_cal / r["ms_cal"] / 1e6, 1)}}
        if "ms_fqpair" in r:
            c["fakequant_pair_metrics"] = {"ms": round(r["ms_fqpair"], 4), "moved_bytes": bytes_fqpair,
                                           "GBps": round(bytes_fqpair / r["ms_fqpair"] / 1e6, 1)}
        else:
            c["fakequant_metrics"] = {"ms": round(r["ms_fq"], 4), "GBps": round(bytes_fq / r["ms_fq"] / 1e6, 1)}
            c["pair_metrics"] = {"ms": round(r["ms_pair"], 4), "GBps": round(bytes_pair / r["ms_pair"] / 1e6, 1)}
        return c

    # dominant kernel: its own algorithmic bytes over its own HIP-event duration
    n_pair_stream = sum(s.numel for s, q in zip(specs, qruns) if q is not None and not
                        (s.scheme == synth.SYM_CHANNEL and s.numel // s.channels <= 8192))
    if args.mode == "single":      # calibration sweep that also compares with qrun: read-only
        kname, kbytes = "k_statspair_stream", 4 * (n_all - n_rowgroup) + 4 * n_pair_stream
    elif args.mode == "fused":
        kname, kbytes = "k_quantpair_stream", bytes_fqpair - 5 * n_rowgroup
    else:
        kname, kbytes = "k_pair_stream", bytes_pair
    kms = main_r["kernels_ms"][kname]
    k_gbps = kbytes / (kms * 1e-3) / 1e9

    out = {
        "metric": "sensitivity_pass_GBps", "value": round(value, 2), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "ms_per_step_median": round(main_r["ms_median"], 4),
        "ms_per_step_min": round(main_r["ms_min"], 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}_b{batch}" + ("_bnfold" if args.fused else ""),
                   "pass": {"single": "qv2_sensitivity_pass: calibrate/fakequant/pair, finalize and rank in one call",
                            "fused": "calibrate + fused fakequant/pair + finalize + rank",
                            "calls": "calibrate + fakequant + pair + finalize + rank"}[args.mode],
                   "tensors": len(specs), "layers": n_layers, "weight_elements": n_w,
                   "activation_elements": n_a, "algorithmic_bytes_per_pass": bytes_pass,
                   "moved_bytes_per_pass": moved, "inputs_checksum": inputs_checksum(specs, xs, qruns, args.checksums)},
        "value_note": "algorithmic bytes of the three calls (4 + 5 + 8 B per element with a partner, fixed "
                      "numerators) / time; it can exceed the HBM rate because the pass visits tensors fewer "
                      "times than three separate calls would. Bytes actually moved / time is hbm_GBps.",
        "paper_context": "the paper reports 2.99-18.99 s per model for its sensitivity list (ResNet50v1: 18.994 s) "
                         "on an Intel i7-12700K + NVIDIA RTX 3090 Ti inside the Glow compiler, including its two "
                         "inferences on real data; another machine and another scope, so no ratio is formed",
        "hbm_GBps": round(moved / (ms_per_step * 1e-3) / 1e9, 2),
        "frac_of_hbm_peak": round(moved / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "layers_per_s": round(n_layers / (ms_per_step * 1e-3), 1),
        "calls": calls_of(main_r), "kernels_ms": main_r["kernels_ms"],
        "roofline": {"bound": "hbm", "kernel": kname, "rocprof_name": ROCPROF_NAMES[kname], "achieved": round(k_gbps, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(k_gbps / HBM_PEAK_GBPS, 4),
                     "traffic": TRAFFIC_BYTES.get(kname) if headline else None,
                     "algorithmic_bytes_per_launch": kbytes, "avg_launch_ms": round(kms, 4)},
        "min_adjacent_score_gap": float(np.min(np.diff(np.sort(last["score"])))) if n_layers > 1 else None,
    }
    # the step after the ranking (Sec. 7, Eq. 17): layers kept in fp32 per BOPs reduction target
    tables = {"resnet50": synth.resnet50_layers, "resnet18": synth.resnet18_layers,
              "vgg16": synth.vgg16_layers, "mobilenetv2": synth.mobilenetv2_layers}
    macs = synth.layer_macs(tables[args.workload]())
    out["bops_cut_layers_kept_fp32"] = {str(t): qb.qv2_bops_select(last["order"], macs, float(t))[1]
                                        for t in (60, 50, 40, 30, 20)}
    if cold_ms is not None:
        out["cold"] = {"ms_per_step": round(cold_ms, 4), "hbm_GBps": round(moved / cold_ms / 1e6, 2),
                       "note": "each step timed alone after a 1 GiB fill; the default figure times steps back to back"}
    if extras:
        out["extras"] = extras
    if other is not None:
        o_bytes = moved_of[other_mode]
        out["other_pass"] = {"pass": "three separate calls" if other_mode == "calls" else "calibrate + fused call",
                             "ms_per_step": round(other["ms_per_step"], 4),
                             "value": round(bytes_pass / other["ms_per_step"] / 1e6, 2),
                             "hbm_GBps": round(o_bytes / other["ms_per_step"] / 1e6, 2),
                             "calls": calls_of(other), "kernels_ms": other["kernels_ms"], "same_order": other["order"] == main_r["order"]}

    if not args.no_cpu_baseline:
        out["cpu_baseline"], out["cpu_baseline_all_cores"] = cpu_baseline(specs, xs, qruns, args.cpu_sample_elems)
        out["oracle_speedup"] = round(value / out["cpu_baseline"]["value"], 1)
    print(json.dumps(out), flush=True)


def inputs_checksum(specs, xs, qruns, verbose):
    """Identity of the synthetic inputs: per tensor the wrapping 64-bit sum of its fp32 bit
    patterns (and of its partner's), combined position-dependently into one hex string.  The
    device generator's stream is not promised stable across torch versions, so runs that are
    to be compared can compare this instead of trusting the seeds."""
    import torch
    acc = 0
    for t, (s, x, q) in enumerate(zip(specs, xs, qruns)):
        cx = int(x.view(-1).view(torch.int32).sum(dtype=torch.int64)) & 0xFFFFFFFFFFFFFFFF
        cq = 0 if q is None else int(q.view(-1).view(torch.int32).sum(dtype=torch.int64)) & 0xFFFFFFFFFFFFFFFF
        if verbose:
            print(f"checksum tensor {t:3d} layer {s.layer:3d} kind {s.kind} numel {s.numel:10d} "
                  f"x {cx:016x} qrun {cq:016x}", file=sys.stderr)
        acc = (acc * 0x100000001B3 + cx) & 0xFFFFFFFFFFFFFFFF
        acc = (acc * 0x100000001B3 + cq) & 0xFFFFFFFFFFFFFFFF
    return f"{acc:016x}"


def cpu_baseline(specs, xs, qruns, budget):
    """The CPU oracle as it stands, timed on a bounded sample of the same workload (tensors
    taken in table order while they fit the element budget): first on one thread, then the same
    unchanged functions with the sample's tensors handed out, largest first, to one thread per
    host core this process may use.  Returns the two records."""
    import os
    from concurrent.futures import ThreadPoolExecutor
    from oracle import reference as orc
    from paper_2501_07161_amd import synth
    orc.lib()
    picked, left = [], budget
    for t, s in enumerate(specs):
        if s.numel <= left:
            picked.append(t)
            left -= s.numel
    host = {t: (xs[t].cpu().numpy().reshape(-1), None if qruns[t] is None else qruns[t].cpu().numpy().reshape(-1))
            for t in picked}

    def one(t):
        s, (x, q) = specs[t], host[t]
        cal = orc.calibrate(x, s.scheme, s.channels)
        fq = orc.fakequant(x, cal, s.scheme, s.channels)
        orc.tensor_metrics(x, cal, fq)
        if q is not None:
            orc.pair_metrics(x, q)
        return (9 if q is None else 17) * x.size

    t0 = time.perf_counter()
    nbytes = sum(one(t) for t in picked)
    dt = time.perf_counter() - t0
    n_w = sum(1 for t in picked if specs[t].kind == synth.WEIGHT)
    sample = (f"{len(picked)} of {len(specs)} tensors of the same workload in table order within "
              f"{budget} elements ({n_w} weights, {len(picked) - n_w} activations with pairs, "
              f"{sum(specs[t].numel for t in picked)} elements)")
    serial = {"value": round(nbytes / dt / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
              "seconds": round(dt, 2), "sample": sample}

    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    env = os.environ.get("OMP_NUM_THREADS", "")
    if env.isdigit() and int(env) > 0:           # the share of the host this job was given
        cores = min(cores, int(env))
    threads = max(1, min(cores, len(picked)))
    by_size = sorted(picked, key=lambda t: -specs[t].numel)
    t0 = time.perf_counter()
    with ThreadPoolExecutor(threads) as pool:    # the oracle's C loops run outside the interpreter lock
        nbytes_mt = sum(pool.map(one, by_size))
    dt_mt = time.perf_counter() - t0
    threaded = {"value": round(nbytes_mt / dt_mt / 1e9, 4), "unit": "GB/s", "cores": threads, "kind": "oracle",
                "seconds": round(dt_mt, 2), "host_cores_visible": os.cpu_count(),
                "sample": sample + "; one tensor per task, largest first, so the largest tensor bounds the time"}
    return serial, threaded


if __name__ == "__main__":
    main()
