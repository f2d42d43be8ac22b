#!/usr/bin/env python3
"""Benchmark of the QuantuneV2 sensitivity pass on one MI355X.

One step = one pass of the whole hot path over the layer table: calibrate
(min/max, statistics, scale, zero-point) -> fake-quantize (int8 codes, error
energies) -> pair metrics (fp32-run vs quantized-run activations) -> fold the
segment records to one per tensor on the device and copy those few KB to the
host -> finalize (MSE, SQNR, mean, var) -> SQNR delta and ranking.  Inputs are
synthetic, seeded, and resident in HBM before the timed region starts.

Workload at N=1: ResNet-50 v1 shapes, batch 256, 224x224 (54 weights,
per-output-channel symmetric; 54 activations with their quantized-run partners,
per-tensor asymmetric).

Prints ONE JSON line.  `value` is the bytes the pass has to move through HBM per
step / time per step, so it is bounded by the HBM rate and `frac_of_hbm_peak` is
value / 8000.  The default pass is the single call (qv2_sensitivity_pass), which
moves 13 B per activation element (x twice - its scale depends on the global
range -, its partner once, one code) and 5 B per element of the per-channel
weights (read once).  Each timed step ends with the sensitivity list on the host
before the next step starts; `pipelined` times the same passes with two in
flight (the host half of one overlaps the device half of the next).  With the
default workload the line also carries `workloads`: the same measurement on the
ResNet-18, MobileNetV2 and VGG-16 sets and on the BN-folded ResNet-50 variant.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X published HBM3E bandwidth
ROCPROF_NAMES = {"k_statspair_stream": "k_stats_stream<512, 8, true, false>",
                 "k_quantpair_stream": "k_quant_stream<256, 2, true, false, true, false>",
                 "k_pair_stream": "k_pair_stream<512, 4>"}
# rocprofv3 --pmc summary of the headline workload; its "traffic_bytes <kernel> <bytes>" lines give the
# HBM bytes per launch (FETCH_SIZE + WRITE_SIZE, each scaled by a copy kernel of known size)
TRAFFIC_PROFILE = os.path.join("profiles", "sensitivity_pass_resnet50_b256.txt")
DEFAULT_BATCH = {"resnet50": 256, "resnet18": 32, "vgg16": 16, "mobilenetv2": 64}


def traffic_from_profile(rocprof_name: str, path: str = None):
    """HBM bytes per launch of a kernel as the committed counter summary states them, or None."""
    path = path or os.path.join(ROOT, TRAFFIC_PROFILE)
    try:
        text = open(path).read()
    except OSError:
        return None
    for m in re.finditer(r"^traffic_bytes\s+(.+?)\s+(\d+)\s*$", text, flags=re.M):
        if m.group(1).strip() == rocprof_name:
            return int(m.group(2))
    return None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="resnet50", choices=["resnet50", "resnet18", "vgg16", "mobilenetv2"])
    ap.add_argument("--batch", type=int, default=None, help="override the workload's batch (smaller = not the headline config)")
    ap.add_argument("--fused", action="store_true", help="BN-folded weight variant of resnet50")
    ap.add_argument("--per-tensor", action="store_true", help="vgg16: per-tensor instead of per-channel weights")
    ap.add_argument("--mode", default="single", choices=["single", "fused", "calls"],
                    help="single: the one call that calibrates, fake-quantizes and compares with the "
                         "quantized run (default); fused: calibrate + fused fake-quant/pair call; "
                         "calls: calibrate, fake-quant and pair as three calls")
    ap.add_argument("--single-mode", action="store_true", help="do not also time the other pass forms and the extras")
    ap.add_argument("--no-workloads", action="store_true",
                    help="default workload only: skip the `workloads` object (the other tensor sets)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--checksums", action="store_true",
                    help="print one checksum line per input tensor to stderr (the JSON line always carries "
                         "their combination as config.inputs_checksum)")
    ap.add_argument("--cpu-sample-elems", type=int, default=0,
                    help="bound the oracle's timing to the first tensors within this many elements "
                         "(0 = every tensor of the workload, streamed one at a time)")
    ap.add_argument("--no-cold", dest="cold", action="store_false",
                    help="skip the second timing in which every step follows a 1 GiB fill that evicts the "
                         "256 MB Infinity Cache (reported as `cold`; it matters only for sets that are not "
                         "far larger than that cache)")
    ap.add_argument("--cold", dest="cold", action="store_true", help="(default) see --no-cold")
    ap.set_defaults(cold=True)
    ap.add_argument("--no-single-tensor-extra", action="store_true",
                    help="skip the 1600 tiny fake-quant calls of extras.fakequant_single_tensor_us (profiling runs)")
    ap.add_argument("--second-read-probe", action="store_true",
                    help="instead of the benchmark: for single tensors of 8 MB ... 800 MB time the quantize sweep "
                         "right after the calibration sweep of the same tensor and again after a 1 GiB fill in "
                         "between (does the second read of x come from the 256 MB memory-side cache?), and a "
                         "read-only sweep repeated on the same tensor; one JSON line.  Run it with the in-tree "
                         "library (non-temporal loads) and with a QV2_NT_LOADS=0 build named by QV2_LIB_PATH")
    ap.add_argument("--copy-probe", action="store_true",
                    help="after the timed region also run 3 plain 1 GiB device copies (a kernel of known "
                         "traffic, used to scale rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    return ap.parse_args()


class Workload:
    """A tensor set resident on the device: specs, tensors, partners, code buffers, layer table."""

    def __init__(self, name, batch, dev, bnfold=False, per_channel=True, share=None):
        import torch
        from paper_2501_07161_amd import binding as qb
        from paper_2501_07161_amd import synth
        self.name, self.batch, self.bnfold = name, batch, bnfold
        if name == "resnet50":
            specs = synth.config_resnet50(batch, fused=bnfold)
        elif name == "vgg16":
            specs = synth.config_vgg16(batch, per_channel=per_channel)
        else:
            specs = synth.CONFIGS[name](batch)
        self.specs = specs
        self.tag = f"{name}_b{batch}" + ("_bnfold" if bnfold else "") + \
            ("_per_tensor" if name == "vgg16" and not per_channel else "")
        # `share`: another workload of the same model and batch whose activations (and their
        # partners and code buffers) are these very tensors - only the weights differ
        reuse = {}
        if share is not None:
            reuse = {s.name: i for i, s in enumerate(share.specs) if s.kind == synth.ACTIVATION}
        xs, qruns, codes, need_q = [], [], [], []
        for i, s in enumerate(specs):
            j = reuse.get(s.name) if s.kind == synth.ACTIVATION else None
            if j is not None:
                xs.append(share.xs[j]); qruns.append(share.qruns[j]); codes.append(share.codes[j])
            else:
                x = synth.materialize(s, dev)
                xs.append(x); qruns.append(None)
                codes.append(torch.empty(x.numel(), dtype=torch.int8, device=dev))
                if s.has_pair:
                    need_q.append(i)
        # quantized-run partners: dequant(quant(ref)) + N(0, (0.01 std(ref))^2).  Built here with
        # the library's own calibrate / fake-quant (untimed set-up) and plain torch arithmetic.
        if need_q:
            rows0 = [qb.TensorArg(x=xs[i], numel=xs[i].numel(), scheme=specs[i].scheme, channels=specs[i].channels,
                                  codes=codes[i]) for i in need_q]
            plan0 = qb.qv2_plan_create(rows0)
            buf0 = qb.Buffers(plan0, dev)
            qb.qv2_calibrate(plan0, buf0.params, buf0.sums, buf0.workspace)
            qb.qv2_fakequant_metrics(plan0, buf0.params, buf0.sums, buf0.workspace)
            torch.cuda.synchronize()
            params, _, _ = buf0.host()
            for k, i in enumerate(need_q):
                p = params[plan0.segment_begin[k]]
                x = xs[i]
                q = codes[i].view(x.shape).to(torch.float32).sub_(float(p["zp"])).mul_(float(p["scale"]))
                q.add_(synth.unit_noise(specs[i], dev), alpha=0.01 * float(x.std(unbiased=False)))
                qruns[i] = q
            plan0.close()
            del buf0
        self.xs, self.qruns, self.codes = xs, qruns, codes
        self.rows = [qb.TensorArg(x=x, numel=x.numel(), scheme=s.scheme, channels=s.channels, qrun=q, codes=c,
                                  kind=s.kind, layer=s.layer) for x, s, q, c in zip(xs, specs, qruns, codes)]
        self.n_layers = max(s.layer for s in specs) + 1
        self.n_w = sum(s.numel for s in specs if s.kind == synth.WEIGHT)
        self.n_a = sum(s.numel for s in specs if s.kind == synth.ACTIVATION)
        self.n_pair = sum(s.numel for s, q in zip(specs, qruns) if q is not None)
        self.n_all = self.n_w + self.n_a
        # elements of the tensors the single call reads once (channels short enough to stay on chip)
        once = []
        for r in self.rows:
            probe = qb.qv2_plan_create([r])
            once.append(probe.num_single_read_elements > 0)
            probe.close()
        self.single_read = once
        self.n_rowgroup = sum(s.numel for s, o in zip(specs, once) if o)
        self.n_pair_stream = sum(s.numel for s, q, o in zip(specs, qruns, once) if q is not None and not o)
        # bytes a pass has to move through HBM, per form
        self.bytes_cal, self.bytes_fq, self.bytes_pair = 4 * self.n_all, 5 * self.n_all, 8 * self.n_pair
        self.bytes_fqpair = 5 * self.n_all + 4 * self.n_pair           # x read once for steps a3 + a4
        self.moved = {"calls": self.bytes_cal + self.bytes_fq + self.bytes_pair,
                      "fused": self.bytes_cal + self.bytes_fqpair,
                      # ... and tensors made of short channels read once for a1 + a3 too
                      "single": self.bytes_cal + self.bytes_fqpair - 4 * self.n_rowgroup}

    def dominant(self, mode):
        """(kernel id name, its algorithmic bytes per launch) of a pass form."""
        if mode == "single":       # calibration sweep that also compares with qrun: read-only
            return "k_statspair_stream", 4 * (self.n_all - self.n_rowgroup) + 4 * self.n_pair_stream
        if mode == "fused":
            return "k_quantpair_stream", self.bytes_fqpair - 5 * self.n_rowgroup
        return "k_pair_stream", self.bytes_pair


class Runner:
    """Plan, buffers and the timed loops of one workload."""

    def __init__(self, wl, dev, steps, warmup):
        import torch
        from paper_2501_07161_amd import binding as qb
        self.wl, self.dev, self.steps, self.warmup = wl, dev, steps, warmup
        self.plan = qb.qv2_plan_create(wl.rows)
        qb.qv2_plan_upload(self.plan)
        self.buf = qb.Buffers(self.plan, dev)
        self.outs = [qb.PassOutputs(self.plan, wl.n_layers, dev) for _ in range(2)]
        self.prep = qb.PreparedPass(self.plan, self.buf.params, self.buf.sums, self.outs, self.buf.workspace)
        qb.qv2_plan_set_timing(self.plan, True)
        self.last = {}
        # the forms made of separate calls bring the records back themselves
        n_ts = self.plan.num_tensors * qb.TENSOR_SUMS.itemsize
        self.d_out = self.outs[0].d_records
        self.d_tsums, self.buf.pair = self.d_out[:n_ts], self.d_out[n_ts:]
        self.h_out = torch.empty(self.d_out.shape, dtype=torch.uint8, pin_memory=True)
        self.h_tsums_np = self.h_out[:n_ts].numpy().view(qb.TENSOR_SUMS)
        self.h_pair_np = self.h_out[n_ts:].numpy().view(qb.PAIR_SUMS)

    def close(self):
        self.plan.close()

    def step(self, mode, events=None):
        import torch
        from paper_2501_07161_amd import binding as qb
        plan, buf = self.plan, self.buf
        if mode == "single":
            # steps 1-4 in ONE native call: device pass, per-tensor fold, one copy of a few KB,
            # Eq. 6-7, Eq. 16 and Algorithm 2; it returns with the list made
            o = self.prep.run()
            self.last.update(order=o.order[:o.n_layers], score=o.score[:o.n_layers])
            return
        if events:
            events[0].record()
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
        qb.qv2_tensor_sums_fold(plan, buf.params, buf.sums, self.d_tsums)
        self.h_out.copy_(self.d_out, non_blocking=True)
        torch.cuda.current_stream().synchronize()
        qb.qv2_finalize_tensors(self.h_tsums_np)                # per tensor: MSE, SQNR, mean, var, absmax
        qb.qv2_pair_finalize(self.h_pair_np)                    # per activation pair: MSE, SQNR
        order, score = qb.qv2_rank_tensors(plan, self.h_tsums_np, self.h_pair_np, self.wl.n_layers)
        self.last.update(order=order, score=score)

    def timed(self, mode):
        """K steps, each complete (list on the host) before the next starts.  The library brackets
        the launches of the form's dominant kernel with HIP events on the call's stream; their
        durations are read after each step."""
        import numpy as np
        import torch
        from paper_2501_07161_amd import binding as qb
        kname, kbytes = self.wl.dominant(mode)
        qb.qv2_plan_time_only(self.plan, kname)
        ev = None
        if mode != "single":
            ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(self.steps)]
        for _ in range(self.warmup):
            self.step(mode)
        torch.cuda.synchronize()
        # a pair of events around a kernel costs a few microseconds of device time: with more than
        # 20 steps the dominant kernel is bracketed in every (steps // 20)-th step of the timed
        # region only, evenly spaced
        stride = max(1, self.steps // 20)
        kms = []
        clock = time.perf_counter
        t0 = clock()
        marks = [t0]
        run_single = self.prep.run if mode == "single" else None
        for k in range(self.steps):
            sampled = k % stride == 0
            if stride > 1 and (sampled or k % stride == 1):
                qb.qv2_plan_set_timing(self.plan, sampled)
            # a step ends with the ranking on the host: it is complete when the call returns
            if run_single is not None:
                run_single()                   # one native call; its outputs are read after the loop
            else:
                self.step(mode, ev[k])
            if sampled:
                kms.append(qb.qv2_plan_kernel_ms(self.plan, kname))
            marks.append(clock())
        torch.cuda.synchronize()
        dt = clock() - t0
        qb.qv2_plan_set_timing(self.plan, True)
        if run_single is not None:
            o = self.outs[0]
            self.last.update(order=o.order[:o.n_layers], score=o.score[:o.n_layers])
        per_step = np.diff(marks) * 1e3
        r = {"ms_per_step": dt / self.steps * 1e3, "ms_median": float(np.median(per_step)),
             "ms_min": float(np.min(per_step)), "order": [int(v) for v in self.last["order"]],
             "kernel": kname, "kernel_bytes": kbytes, "kernel_ms": float(np.mean(kms)),
             "kernel_launches_timed": len(kms)}
        if mode == "fused":
            r["ms_cal"] = float(np.mean([e[0].elapsed_time(e[1]) for e in ev]))
            r["ms_fqpair"] = float(np.mean([e[1].elapsed_time(e[3]) for e in ev]))
        elif mode == "calls":
            r["ms_cal"] = float(np.mean([e[0].elapsed_time(e[1]) for e in ev]))
            r["ms_fq"] = float(np.mean([e[1].elapsed_time(e[2]) for e in ev]))
            r["ms_pair"] = float(np.mean([e[2].elapsed_time(e[3]) for e in ev]))
        return r

    def all_kernels_ms(self, mode, reps=5):
        """Per-kernel durations of a form (every tile kernel bracketed; not part of a timed loop)."""
        import numpy as np
        import torch
        from paper_2501_07161_amd import binding as qb
        names = {"single": ["k_statspair_stream", "k_quant_stream", "k_single_read_rows"],
                 "fused": ["k_stats_stream", "k_stats_rows", "k_quantpair_stream", "k_quantpair_rows"],
                 "calls": ["k_stats_stream", "k_stats_rows", "k_quant_stream", "k_quant_rows", "k_pair_stream"]}[mode]
        qb.qv2_plan_time_only(self.plan, None)
        rows = []
        for _ in range(reps):
            self.step(mode)
            torch.cuda.synchronize()
            rows.append(qb.qv2_plan_kernels_ms(self.plan).copy())
        return {n: round(float(np.mean([r[qb.KERNEL_IDS[n]] for r in rows])), 4) for n in names}

    def timed_pipelined(self):
        """The same K passes with two in flight: pass k+1 is enqueued before the host waits for
        pass k's records and ranks them.  Every pass still does all of its work and its list is
        made on the host; only the waiting overlaps.  No events inside the passes."""
        import torch
        from paper_2501_07161_amd import binding as qb
        qb.qv2_plan_set_timing(self.plan, False)
        prep = self.prep
        for k in range(max(2, self.warmup)):
            prep.begin(k & 1)
            prep.end(k & 1)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        prep.begin(0)
        for k in range(1, self.steps):
            prep.begin(k & 1)
            prep.end((k - 1) & 1)
        o = prep.end((self.steps - 1) & 1)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        qb.qv2_plan_set_timing(self.plan, True)
        return {"ms_per_step": dt / self.steps * 1e3, "order": [int(v) for v in o.order[:o.n_layers]]}

    def cold(self, mode):
        import numpy as np
        import torch
        scratch = torch.empty(1 << 28, dtype=torch.float32, device=self.dev)
        ts = []
        for _ in range(self.steps):
            scratch.fill_(1.0)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            self.step(mode)
            torch.cuda.synchronize()
            ts.append(time.perf_counter() - t0)
        return float(np.mean(ts)) * 1e3


def second_read_probe(dev):
    """Per tensor size: the calibration sweep, then the quantize sweep of the same tensor, (warm) back
    to back, (cold) with a 1 GiB fill between the two, (requant) the quantize sweep alone repeated;
    and the calibration sweep alone repeated.  Kernel durations from the library's HIP events."""
    import numpy as np
    import torch
    from paper_2501_07161_amd import binding as qb
    flush = torch.empty(1 << 28, dtype=torch.float32, device=dev)
    out = {"library": os.path.basename(qb.LIB_PATH), "sizes": {}}
    for mb in (8, 16, 32, 64, 96, 128, 160, 200, 256, 400, 800):
        n = mb * 1024 * 1024 // 4
        x = torch.randn(n, device=dev).clamp_(min=0)
        c = torch.empty(n, dtype=torch.int8, device=dev)
        plan = qb.qv2_plan_create([qb.TensorArg(x=x, numel=n, codes=c)])
        buf = qb.Buffers(plan, dev)
        qb.qv2_plan_set_timing(plan, True)
        rec = {}
        for mode in ("warm", "cold", "requant"):
            ts, tq = [], []
            for it in range(8):
                if mode != "requant":
                    flush.fill_(1.0)
                    qb.qv2_calibrate(plan, buf.params, buf.sums, buf.workspace)
                if mode == "cold":
                    flush.fill_(1.0)
                qb.qv2_fakequant_metrics(plan, buf.params, buf.sums, buf.workspace)
                torch.cuda.synchronize()
                if it >= 2:
                    ts.append(qb.qv2_plan_kernel_ms(plan, "k_stats_stream"))
                    tq.append(qb.qv2_plan_kernel_ms(plan, "k_quant_stream"))
            rec[mode] = {"stats_us": round(float(np.median(ts)) * 1e3, 1), "quant_us": round(float(np.median(tq)) * 1e3, 1)}
        ts = []
        for it in range(8):
            qb.qv2_calibrate(plan, buf.params, buf.sums, buf.workspace)
            torch.cuda.synchronize()
            if it >= 2:
                ts.append(qb.qv2_plan_kernel_ms(plan, "k_stats_stream"))
        rec["restats_us"] = round(float(np.median(ts)) * 1e3, 1)
        out["sizes"][f"{mb}MB"] = rec
        plan.close()
        del x, c, buf
    return out


def gbps(nbytes, ms):
    return nbytes / (ms * 1e-3) / 1e9 if ms > 0 else 0.0


def summarize(wl, r, pipe, mode):
    """The record of one workload in one pass form: step time, bytes moved, fraction of the HBM
    peak, and the same for its dominant kernel."""
    moved = wl.moved[mode]
    k_rate = gbps(r["kernel_bytes"], r["kernel_ms"]) if r["kernel_ms"] > 0 else 0.0
    out = {"ms_per_step": round(r["ms_per_step"], 4), "ms_per_step_median": round(r["ms_median"], 4),
           "ms_per_step_min": round(r["ms_min"], 4), "moved_bytes_per_pass": moved,
           "GBps": round(gbps(moved, r["ms_per_step"]), 2),
           "frac_of_hbm_peak": round(gbps(moved, r["ms_per_step"]) / HBM_PEAK_GBPS, 4),
           "tensors": len(wl.specs), "layers": wl.n_layers,
           "dominant_kernel": {"kernel": r["kernel"], "avg_launch_ms": round(r["kernel_ms"], 4),
                               "launches_timed": r["kernel_launches_timed"],
                               "algorithmic_bytes_per_launch": r["kernel_bytes"], "GBps": round(k_rate, 1),
                               "frac": round(k_rate / HBM_PEAK_GBPS, 4)}}
    if pipe is not None:
        out["pipelined"] = {"ms_per_step": round(pipe["ms_per_step"], 4),
                            "GBps": round(gbps(moved, pipe["ms_per_step"]), 2),
                            "frac_of_hbm_peak": round(gbps(moved, pipe["ms_per_step"]) / HBM_PEAK_GBPS, 4),
                            "same_order": pipe["order"] == r["order"]}
    return out


def side_workloads(args, dev, head):
    """The other tensor sets of the evaluation (and the BN-folded weights of the headline set), each
    through the same measurement: single call serial and pipelined, dominant kernel, and the list
    of the three-call form for comparison."""
    import torch
    out = {}
    todo = [("resnet18", {}), ("mobilenetv2", {}), ("vgg16", {"per_channel": True}),
            ("vgg16", {"per_channel": False}), ("resnet50", {"bnfold": True, "share": head})]
    for name, kw in todo:
        wl = Workload(name, DEFAULT_BATCH[name], dev, **kw)
        # a pass over these sets takes a fraction of a millisecond: ten times the steps, so that the
        # timed region is not a few milliseconds of a clock that is still ramping
        steps = args.steps * (1 if kw.get("bnfold") else 10)
        rn = Runner(wl, dev, steps, args.warmup)
        r = rn.timed("single")
        pipe = rn.timed_pipelined()
        rec = summarize(wl, r, pipe, "single")
        rec["steps"] = steps
        rn.step("calls")
        rec["same_order_as_three_calls"] = [int(v) for v in rn.last["order"]] == r["order"]
        out[wl.tag] = rec
        rn.close()
        del rn, wl
        torch.cuda.empty_cache()
    return out


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

    if args.second_read_probe:
        print(json.dumps(second_read_probe(dev)), flush=True)
        return

    batch = args.batch or DEFAULT_BATCH[args.workload]
    wl = Workload(args.workload, batch, dev, bnfold=args.fused, per_channel=not args.per_tensor)
    headline = args.workload == "resnet50" and batch == 256 and not args.fused
    rn = Runner(wl, dev, args.steps, args.warmup)
    plan, buf = rn.plan, rn.buf
    specs, n_layers = wl.specs, wl.n_layers

    main_r = rn.timed(args.mode)
    pipe = rn.timed_pipelined() if args.mode == "single" else None
    kernels_ms = rn.all_kernels_ms(args.mode)
    cold_ms = rn.cold(args.mode) if args.cold else None
    other_mode = "fused" if args.mode == "calls" else "calls"
    other = None if args.single_mode else rn.timed(other_mode)
    if other is not None:
        other["kernels_ms"] = rn.all_kernels_ms(other_mode)
    score = np.array(rn.last["score"], dtype=np.float64)
    qb.qv2_plan_time_only(plan, None)

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
                               kind=r.kind, layer=r.layer) for r in wl.rows]
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
        hist_bytes = 4 * wl.n_all + 4 * wl.n_pair
        moved_m = 8 * wl.n_all + 4 * wl.n_pair - 4 * wl.n_rowgroup
        extras = {"histogram_2048_bins": {"kernel_ms": round(float(np.mean(t_h)), 4),
                                          "GBps": round(hist_bytes / np.mean(t_h) / 1e6, 1)},
                  "fused_quantize_with_cosine": {"kernel_ms": round(float(np.mean(t_c)), 4)},
                  "single_call_with_cosine": {"call_ms": round(float(np.mean(t_s)), 4)},
                  "single_call_metrics_only": {"call_ms": round(float(np.mean(t_m)), 4), "moved_bytes": moved_m,
                                               "GBps": round(moved_m / np.mean(t_m) / 1e6, 1)}}
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

    workloads = None
    if headline and not args.no_workloads and args.mode == "single":
        rn.close()                               # the side sets need no plan of the headline set
        workloads = side_workloads(args, dev, wl)

    ms_per_step = main_r["ms_per_step"]
    moved = wl.moved[args.mode]
    value = gbps(moved, ms_per_step)
    three_call_bytes = wl.moved["calls"]

    def calls_of(r):
        if "ms_cal" not in r:       # one host call that also waits, finalizes and ranks
            return {"sensitivity_pass": {"ms": round(r["ms_per_step"], 4), "moved_bytes": wl.moved["single"],
                                         "GBps": round(gbps(wl.moved["single"], r["ms_per_step"]), 1)}}
        c = {"calibrate": {"ms": round(r["ms_cal"], 4), "GBps": round(gbps(wl.bytes_cal, r["ms_cal"]), 1)}}
        if "ms_fqpair" in r:
            c["fakequant_pair_metrics"] = {"ms": round(r["ms_fqpair"], 4), "moved_bytes": wl.bytes_fqpair,
                                           "GBps": round(gbps(wl.bytes_fqpair, r["ms_fqpair"]), 1)}
        else:
            c["fakequant_metrics"] = {"ms": round(r["ms_fq"], 4), "GBps": round(gbps(wl.bytes_fq, r["ms_fq"]), 1)}
            c["pair_metrics"] = {"ms": round(r["ms_pair"], 4), "GBps": round(gbps(wl.bytes_pair, r["ms_pair"]), 1)}
        return c

    # dominant kernel: its own algorithmic bytes over its own HIP-event duration in the timed steps
    kname, kbytes, kms = main_r["kernel"], main_r["kernel_bytes"], main_r["kernel_ms"]
    k_gbps = gbps(kbytes, kms)
    traffic = traffic_from_profile(ROCPROF_NAMES[kname]) if headline else None

    out = {
        "metric": "sensitivity_pass_GBps", "value": round(value, 2), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "ms_per_step_median": round(main_r["ms_median"], 4),
        "ms_per_step_min": round(main_r["ms_min"], 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.tag,
                   "pass": {"single": "qv2_sensitivity_pass: calibrate/fakequant/pair, finalize and rank in one call",
                            "fused": "calibrate + fused fakequant/pair + finalize + rank",
                            "calls": "calibrate + fakequant + pair + finalize + rank"}[args.mode],
                   "tensors": len(specs), "layers": n_layers, "weight_elements": wl.n_w,
                   "activation_elements": wl.n_a, "moved_bytes_per_pass": moved,
                   "three_call_bytes_per_pass": three_call_bytes,
                   "inputs_checksum": inputs_checksum(specs, wl.xs, wl.qruns, args.checksums)},
        "value_note": "bytes this pass form has to move through HBM per step (single call: 13 B per activation "
                      "element, 5 B per element of a per-channel weight read once) / time per step; each step ends "
                      "with the sensitivity list on the host before the next begins",
        "frac_of_hbm_peak": round(value / HBM_PEAK_GBPS, 4),
        "three_call_equivalent_GBps": round(gbps(three_call_bytes, ms_per_step), 2),
        "three_call_equivalent_note": "4 + 5 + 8 B per element with a partner (calibrate, fake-quant and pair as "
                                      "three separate visits) / the same time: what three calls would have to sustain "
                                      "to finish as fast; not an HBM rate, it may exceed the peak",
        "paper_context": "the paper reports 2.99-18.99 s per model for its sensitivity list (ResNet50v1: 18.994 s) "
                         "on an Intel i7-12700K + NVIDIA RTX 3090 Ti inside the Glow compiler, including its two "
                         "inferences on real data; another machine and another scope, so no ratio is formed",
        "layers_per_s": round(n_layers / (ms_per_step * 1e-3), 1),
        "calls": calls_of(main_r), "kernels_ms": kernels_ms,
        "roofline": {"bound": "hbm", "kernel": kname, "rocprof_name": ROCPROF_NAMES[kname], "achieved": round(k_gbps, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(k_gbps / HBM_PEAK_GBPS, 4),
                     "traffic": traffic, "traffic_source": TRAFFIC_PROFILE if traffic is not None else None,
                     "algorithmic_bytes_per_launch": kbytes, "avg_launch_ms": round(kms, 4),
                     "launches_timed": main_r["kernel_launches_timed"]},
        "min_adjacent_score_gap": float(np.min(np.diff(np.sort(score)))) if n_layers > 1 else None,
    }
    if pipe is not None:
        out["pipelined"] = {"ms_per_step": round(pipe["ms_per_step"], 4),
                            "GBps": round(gbps(moved, pipe["ms_per_step"]), 2),
                            "frac_of_hbm_peak": round(gbps(moved, pipe["ms_per_step"]) / HBM_PEAK_GBPS, 4),
                            "same_order": pipe["order"] == main_r["order"],
                            "note": "the same passes with two in flight (qv2_sensitivity_pass_begin / _end): the "
                                    "host half of a pass overlaps the device half of the next"}
    # the step after the ranking (Sec. 7, Eq. 17): layers kept in fp32 per BOPs reduction target
    tables = {"resnet50": synth.resnet50_layers, "resnet18": synth.resnet18_layers,
              "vgg16": synth.vgg16_layers, "mobilenetv2": synth.mobilenetv2_layers}
    macs = synth.layer_macs(tables[args.workload]())
    out["bops_cut_layers_kept_fp32"] = {str(t): qb.qv2_bops_select(main_r["order"], macs, float(t))[1]
                                        for t in (60, 50, 40, 30, 20)}
    if cold_ms is not None:
        out["cold"] = {"ms_per_step": round(cold_ms, 4), "GBps": round(gbps(moved, cold_ms), 2),
                       "note": "each step timed alone after a 1 GiB fill; the default figure times steps back to back"}
    if extras:
        out["extras"] = extras
    if other is not None:
        out["other_pass"] = {"pass": "three separate calls" if other_mode == "calls" else "calibrate + fused call",
                             "ms_per_step": round(other["ms_per_step"], 4),
                             "GBps": round(gbps(wl.moved[other_mode], other["ms_per_step"]), 2),
                             "moved_bytes_per_pass": wl.moved[other_mode],
                             "calls": calls_of(other), "kernels_ms": other["kernels_ms"],
                             "same_order": other["order"] == main_r["order"]}
    if workloads is not None:
        out["workloads"] = workloads

    if not args.no_cpu_baseline:
        serial, threaded = cpu_baseline(wl, args.cpu_sample_elems)
        out["cpu_baseline"], out["cpu_baseline_all_cores"] = serial, threaded
        # the same tensors on both sides: seconds the oracle needs for them / seconds the pass needs
        share = serial["elements_covered"] / serial["elements_total"]
        gpu_s = ms_per_step * 1e-3
        out["oracle_speedup"] = {"vs_1_core": round(serial["seconds"] / (gpu_s * share), 1),
                                 "vs_all_cores": round(threaded["seconds"] / (gpu_s * threaded["elements_covered"]
                                                                              / threaded["elements_total"]), 1),
                                 "cores": threaded["cores"],
                                 "basis": "oracle seconds for the covered tensors / pass seconds scaled to the same "
                                          "share of the workload's elements"}
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


def cpu_baseline(wl, budget):
    """The CPU oracle as it stands, timed on the tensors of the same workload: first on one
    thread, tensor after tensor (each copied from the device just before its turn, so the host
    holds one tensor and its partner at a time), then the same unchanged functions with the
    tensors handed out, largest first, to one thread per host core this process may use (in
    batches of a few GB of host copies).  Only the oracle calls are timed, not the copies.
    budget > 0 bounds both legs to the first tensors in table order that fit that many elements.
    The rate is in the pass's own unit: the bytes the GPU pass moves for the covered tensors
    (13 B per element with a partner, 9 B without, 5 B for a tensor made of short channels) over
    the oracle's seconds."""
    from concurrent.futures import ThreadPoolExecutor
    from oracle import reference as orc
    from paper_2501_07161_amd import synth
    orc.lib()
    specs, xs, qruns = wl.specs, wl.xs, wl.qruns
    total = sum(s.numel for s in specs)
    if budget and budget > 0:
        picked, left = [], budget
        for t, s in enumerate(specs):
            if s.numel <= left:
                picked.append(t)
                left -= s.numel
    else:
        picked = list(range(len(specs)))
    covered = sum(specs[t].numel for t in picked)

    def fetch(t):
        return (xs[t].cpu().numpy().reshape(-1), None if qruns[t] is None else qruns[t].cpu().numpy().reshape(-1))

    def moved_bytes(t):
        s = specs[t]
        return (5 if wl.single_read[t] else 9) * s.numel + (4 * s.numel if qruns[t] is not None else 0)

    def one(t, x, q):
        s = specs[t]
        cal = orc.calibrate(x, s.scheme, s.channels)
        fq = orc.fakequant(x, cal, s.scheme, s.channels)
        orc.tensor_metrics(x, cal, fq)
        if q is not None:
            orc.pair_metrics(x, q)

    nbytes = sum(moved_bytes(t) for t in picked)
    dt = 0.0
    for t in picked:
        x, q = fetch(t)
        t0 = time.perf_counter()
        one(t, x, q)
        dt += time.perf_counter() - t0
        del x, q
    n_w = sum(1 for t in picked if specs[t].kind == synth.WEIGHT)
    sample = (f"{len(picked)} of {len(specs)} tensors of the same workload ({n_w} weights, "
              f"{len(picked) - n_w} activations), {covered} of {total} elements")
    serial = {"value": round(nbytes / dt / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
              "seconds": round(dt, 2), "elements_covered": covered, "elements_total": total, "sample": sample}

    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    env = os.environ.get("OMP_NUM_THREADS", "")
    if env.isdigit() and int(env) > 0:           # the share of the host this job was given
        cores = min(cores, int(env))
    threads = max(1, min(cores, len(picked)))
    by_size = sorted(picked, key=lambda t: -specs[t].numel)
    dt_mt, i = 0.0, 0
    with ThreadPoolExecutor(threads) as pool:    # the oracle's C loops run outside the interpreter lock
        while i < len(by_size):
            batch, held = [], 0
            while i < len(by_size) and (len(batch) < threads or held < (1 << 30)) and held < (3 << 30) // 2:
                t = by_size[i]
                batch.append((t,) + fetch(t))
                held += specs[t].numel
                i += 1
            t0 = time.perf_counter()
            list(pool.map(lambda a: one(*a), batch))
            dt_mt += time.perf_counter() - t0
            del batch
    threaded = {"value": round(nbytes / dt_mt / 1e9, 4), "unit": "GB/s", "cores": threads, "kind": "oracle",
                "seconds": round(dt_mt, 2), "elements_covered": covered, "elements_total": total,
                "host_cores_visible": os.cpu_count(),
                "sample": sample + "; one tensor per task, largest first, in batches of at most 1.5 G elements"}
    return serial, threaded


if __name__ == "__main__":
    main()
