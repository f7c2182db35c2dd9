#!/usr/bin/env python3
"""Benchmark of the MoE expert FFN layer on one MI355X.

A step is one pass of the whole hot path (gate -> permute -> grouped FFN -> combine) over one
batch of seeded synthetic tokens, with inputs and quantised weights already resident in HBM.
Prints ONE JSON line: whole-job tokens/s of the headline workload (c2, the decode-like,
bandwidth-bound configuration), the roofline figures of its dominant kernel (the grouped
weight-quantised GEMM) from HIP events, the CPU oracle timed beside it, and, under
"other_workloads", the same figures for the remaining configurations (c1, c3, c4, c5 with fp16
and with bf16 rows), each with a roofline block of its own.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2] [--no-cpu-baseline] [--no-others]

Cold-cache protocol: the weights of the small workloads would fit in the 256 MB last-level
cache, so the layer cycles through a ring of identical weight copies (>= 1 GiB in total), one
copy per step; every step therefore streams its weights from HBM.
"""
from __future__ import annotations

import argparse
import gc
import glob
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_F16_PEAK_TFLOPS = 2500.0  # MI355X dense fp16 MFMA, published
OTHERS = ["c1", "c3", "c4", "c5", "c5_bf16"]


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="leave out the other_workloads block (the headline workload only)")
    ap.add_argument("--ring-bytes", type=float, default=float(1 << 30))
    ap.add_argument("--finished", type=float, default=0.0,
                    help="fraction of the rows marked finished (batch pruning, Sec. 3.5); 0 = the headline workload")
    ap.add_argument("--traffic-calibration", action="store_true",
                    help="also run 5 plain device copies of 256 MiB: under `rocprofv3 --pmc FETCH_SIZE|WRITE_SIZE` "
                         "their counter reading calibrates the bytes-per-count of the GEMM's reading")
    return ap.parse_args()


def describe(w):
    q = "int%d %s" % (w.bits, "per-channel" if w.group_size == 0 else "group-%d" % w.group_size)
    return "%s: T=%d d_model=%d d_ff=%d E=%d top-%d %s act=%s seed=%d" % (
        w.name, w.T, w.d, w.F, w.E, w.k, q, w.act, w.seed)


def measured_traffic(workload: str, kernels: str):
    """HBM bytes per GEMM launch from the rocprofv3 counter summaries under profiles/: the line
    `roofline.traffic[<workload>] = <bytes> bytes per launch, kernel <name>` of the summary that
    covers this workload.  None when no summary names the kernel that ran."""
    pat = re.compile(r"roofline\.traffic\[(\w+)\]\s*=\s*([0-9.eE+]+)\s*bytes per launch,\s*kernel\s+(\w+)")
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.md"))):
        for m in pat.finditer(open(path).read()):
            if m.group(1) == workload and m.group(3) in kernels.split():
                return float(m.group(2)), os.path.relpath(path, ROOT)
    return None, None


def box_peaks(torch, binding):
    """The peaks re-derived from what the box reports (CUs x 4096 fp16 flop per clock x engine
    clock; memory bus width x pin rate, the pin rate of HBM3E being four transfers per reported
    memory clock: 8 Gbit/s at the 2000 MHz this chip reports), printed beside the published constants."""
    p = torch.cuda.get_device_properties(0)
    info = binding.moe_device_info()
    cus, clk, mclk, bus = info["compute_units"], info["engine_clock_khz"], info["memory_clock_khz"], info["memory_bus_bits"]
    out = {"device": p.name, "arch": getattr(p, "gcnArchName", None), "compute_units": cus,
           "engine_clock_mhz": None if clk is None else clk / 1e3,
           "memory_clock_mhz": None if mclk is None else mclk / 1e3, "memory_bus_bits": bus,
           "mfma_f16_tflops_derived": None, "hbm_gbs_derived": None,
           "mfma_f16_tflops_published": MFMA_F16_PEAK_TFLOPS, "hbm_gbs_published": HBM_PEAK_GBS}
    if cus and clk:
        out["mfma_f16_tflops_derived"] = cus * 4096 * clk * 1e3 / 1e12
    if mclk and bus:
        out["hbm_gbs_derived"] = mclk * 1e3 * 4 * bus / 8 / 1e9
    return out


def stats_us(ms):
    import numpy as np
    a = np.asarray(ms, dtype=np.float64) * 1e3
    return {"median": float(np.median(a)), "min": float(a.min()), "mean": float(a.mean())}


def measure(name, args, cpu_baseline, headline):
    """Builds the layer of one workload, times K whole steps and, in a second pass of K steps, every
    step of the path between HIP events.  Returns the result fields of that workload."""
    import numpy as np
    import torch

    from paper_2211_10017_amd import MoEExpertLayer, binding
    from paper_2211_10017_amd import workloads as W

    w = W.WORKLOADS[name]
    dev = "cuda:0"
    tdt = torch.float16 if w.act == "f16" else torch.bfloat16
    layer = MoEExpertLayer(w.T, w.d, w.F, w.E, w.k, w.bits, w.group_size, act_dtype=tdt,
                           renormalize=w.renormalize, device=dev)
    x_np, wg_np, bias_np = W.activations(w), W.gate_weight(w), W.gate_bias(w)
    layer.wg.copy_(torch.from_numpy(wg_np).to(dev, tdt))
    if bias_np is not None:
        layer.gate_bias = torch.from_numpy(bias_np).to(dev)
    x = torch.from_numpy(x_np).to(dev, tdt)
    keep_masters = cpu_baseline and w.E * w.d * w.F * 8 <= 4e9
    masters = {1: [], 2: []}
    for which in (1, 2):
        for e0, ms in W.expert_weight_batches(w, which, threads=16):
            for i, m in enumerate(ms):
                layer.load_expert(which, e0 + i, torch.from_numpy(m).to(dev))
                if keep_masters:
                    masters[which].append(m)
    torch.cuda.synchronize()

    # ring of weight copies so that every step reads its weights from HBM, not from cache
    wbytes = layer.w1_packed.numel() + layer.w2_packed.numel() + 2 * (layer.s1.numel() + layer.s2.numel())
    ncopy = max(1, min(64, int(-(-args.ring_bytes // wbytes))))
    ring = [(layer.w1_packed, layer.s1, layer.w2_packed, layer.s2)]
    for _ in range(ncopy - 1):
        ring.append(tuple(t.clone() for t in ring[0]))

    finished = None
    if args.finished > 0:
        mask = np.random.default_rng(w.seed + 100).random(w.T) < args.finished
        finished = torch.from_numpy(mask.astype(np.uint8)).to(dev)

    def step(i):
        layer.w1_packed, layer.s1, layer.w2_packed, layer.s2 = ring[i % ncopy]
        layer.forward(x, finished)

    steps = args.steps
    for i in range(ncopy):                # first use of every ring copy marshals its argument lists: not a step
        step(i)
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / steps * 1e3
    tokens_per_s = w.T * steps / elapsed
    kernels = binding.load().moe_last_ffn_kernels().decode()      # what the library launched for the GEMM pair

    # ---- the grouped FFN alone, K calls back to back between two HIP events (on torch's current stream,
    # which is the stream the library launches on): the roofline's timing.  Routing state is that of
    # the last step; every call streams another ring copy of the weights.  Event pairs around single
    # calls would add the events' own cost (several microseconds, see step_us.empty_interval) to a
    # call that takes tens of microseconds.
    reps = 5
    evf = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in evf:
        a.record()
        for i in range(steps):
            layer.w1_packed, layer.s1, layer.w2_packed, layer.s2 = ring[i % ncopy]
            layer.ffn(x, finished)
        b.record()
    torch.cuda.synchronize()
    # ---- where the FFN call is the decode kernel plus its small slice reduction: the decode kernel alone,
    # the same way (the gated call with a NULL output leaves the reduction out).  The roofline is that
    # kernel's; the whole call's time is reported beside it.
    kernel_ms = None
    if kernels.split()[:1] == ["decode_ffn_kernel"]:
        evk = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for a, b in evk:
            a.record()
            for i in range(steps):
                layer.w1_packed, layer.s1, layer.w2_packed, layer.s2 = ring[i % ncopy]
                layer.ffn_streaming_kernel_only(x, finished)
            b.record()
        torch.cuda.synchronize()
        kernel_ms = np.array([a.elapsed_time(b) / steps for a, b in evk])
        layer.ffn(x, finished)                            # (leaves `out` and the kernel notes as a full call does)
    # ---- and once more with an event between all steps of the path: median and minimum of each step
    names = ["gate", "permute", "ffn", "combine"]
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(steps)]
    for i in range(steps):
        layer.w1_packed, layer.s1, layer.w2_packed, layer.s2 = ring[i % ncopy]
        ev[i][0].record()
        layer.gate(x, finished)
        ev[i][1].record()
        layer.permute(x, finished)
        ev[i][2].record()
        layer.ffn(x, finished)
        ev[i][3].record()
        layer.combine(x, finished)
        ev[i][4].record()
    torch.cuda.synchronize()
    per_step = {n: stats_us([e[j].elapsed_time(e[j + 1]) for e in ev]) for j, n in enumerate(names)}
    per_step["chain"] = stats_us([e[0].elapsed_time(e[4]) for e in ev])
    # what a pair of events reads with nothing between them: every interval above contains this much
    # that is not kernel time (a step that a fused entry point absorbed reads about this value)
    idle = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for a, b in idle:
        a.record()
        b.record()
    torch.cuda.synchronize()
    per_step["empty_interval"] = stats_us([a.elapsed_time(b) for a, b in idle])
    planned = [what for _, _, what in layer._plan(x, finished)]
    per_step["launch_sequence"] = planned            # a step the fused entry points absorbed shows ~0 us above
    ffn_ms = np.array([a.elapsed_time(b) / steps for a, b in evf])     # per call, each averaged over K calls
    # fc1 and fc2 are two launches of the GEMM kernel, except in the decode kernel, which streams both
    # weight matrices in one launch and is timed without its slice reduction
    launches_per_ffn = max(1, len(kernels.split()))
    launch_s = float((ffn_ms if kernel_ms is None else kernel_ms).mean()) * 1e-3 / launches_per_ffn

    if args.traffic_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()

    off = layer.expert_offsets.cpu().numpy()
    active = int((np.diff(off) > 0).sum())
    active_rows = int(off[w.E])
    g1 = w.d if w.group_size in (0, w.d) else w.group_size
    g2 = w.F if w.group_size in (0, w.F) else w.group_size
    # algorithmic bytes: codes and fp16 scales of the experts that received rows
    bytes_ffn = active * (2 * w.d * w.F * w.bits // 8 + 2 * ((w.d // g1) * w.F + (w.F // g2) * w.d))
    flops_ffn = 4.0 * active_rows * w.d * w.F
    intensity = flops_ffn / bytes_ffn
    if intensity < MFMA_F16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9):
        achieved = bytes_ffn / launches_per_ffn / launch_s / 1e9
        roofline = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": achieved / HBM_PEAK_GBS, "traffic": None}
    else:
        achieved = flops_ffn / launches_per_ffn / launch_s / 1e12
        roofline = {"bound": "mfma", "achieved": achieved, "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": achieved / MFMA_F16_PEAK_TFLOPS, "traffic": None}
    traffic, source = measured_traffic(w.name, kernels) if args.finished == 0 else (None, None)
    roofline["traffic"] = traffic
    roofline.update({"traffic_source": source, "kernel": kernels.split()[0] if kernels else None, "kernels_launched": kernels,
                     "launches_per_step": launches_per_ffn,
                     "avg_launch_us": launch_s * 1e6, "ffn_call_us_mean": float(ffn_ms.mean()) * 1e3,
                     "ffn_call_us_min": float(ffn_ms.min()) * 1e3,
                     "ffn_call_frac": (bytes_ffn / (float(ffn_ms.mean()) * 1e-3) / 1e9 / HBM_PEAK_GBS
                                       if roofline["bound"] == "hbm" else flops_ffn / (float(ffn_ms.mean()) * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS),
                     "timing": ("%d x %d back-to-back launches of the kernel alone (FFN call without its slice reduction) between HIP events"
                                if kernel_ms is not None else "%d x %d back-to-back FFN calls between HIP events") % (reps, steps),
                     "active_experts": active,
                     "algorithmic_bytes_per_step": int(bytes_ffn), "flops_per_step": flops_ffn,
                     "weight_ring_copies": ncopy})

    result = {
        "value": tokens_per_s, "unit": "tokens/s", "ms_per_step": ms_per_step, "steps": steps, "dtype": w.act,
        "config": {"workload": describe(w), "weights": "int%d" % w.bits,
                   "routed_rows": w.R, "cold_weights": ncopy > 1,
                   **({"finished_fraction": args.finished, "active_rows": active_rows}
                      if args.finished > 0 else {})},
        "roofline": roofline, "step_us": per_step,
    }

    # ---- the CPU oracle on the same inputs, on this machine's host cores (a reported baseline)
    if cpu_baseline:
        import oracle
        act = oracle.F16 if w.act == "f16" else oracle.BF16
        if keep_masters:
            q1, s1 = oracle.quantize(np.stack(masters[1]), w.bits, w.group_size)
            q2, s2 = oracle.quantize(np.stack(masters[2]), w.bits, w.group_size)

            def timed(budget_s, most):
                reps, spent = 0, 0.0
                while spent < budget_s and reps < most:
                    t0 = time.perf_counter()
                    oracle.moe_layer(x_np, wg_np, bias_np, q1, s1, q2, s2, w.k, w.group_size, act,
                                     renormalize=w.renormalize)
                    spent += time.perf_counter() - t0
                    reps += 1
                return reps, spent

            cores = oracle.num_threads()
            reps, spent = timed(10.0 if headline else 4.0, 50)
            result["cpu_baseline"] = {"value": w.T * reps / spent, "unit": "tokens/s",
                                      "cores": cores, "kind": "oracle",
                                      "sample": "%d full passes of the same layer (all %d tokens), %.1f s" % (reps, w.T, spent)}
            oracle.set_num_threads(1)             # the same passes on one core
            reps1, spent1 = timed(6.0 if headline else 3.0, 10)
            oracle.set_num_threads(cores)
            result["cpu_baseline"]["single_thread"] = {"value": w.T * reps1 / spent1, "unit": "tokens/s", "cores": 1,
                                                       "sample": "%d full passes, %.1f s" % (reps1, spent1)}
        else:
            # too large to keep on the host: time the oracle's expert FFN on a sample of rows of
            # expert 0 and scale to the routed rows of the layer (rows are independent)
            m1, m2 = W.expert_weight(w, 1, 0), W.expert_weight(w, 2, 0)
            q1, s1 = oracle.quantize(m1[None], w.bits, w.group_size)
            q2, s2 = oracle.quantize(m2[None], w.bits, w.group_size)
            rows = max(oracle.num_threads(), 16)
            xs = np.tile(x_np, (-(-rows // w.T), 1))[:rows]
            t0 = time.perf_counter()
            w1 = oracle.dequantize(q1, s1, w.group_size)[0]
            w2 = oracle.dequantize(q2, s2, w.group_size)[0]
            t_deq = time.perf_counter() - t0
            t0 = time.perf_counter()
            oracle.expert_ffn(xs, w1, w2, act)
            t_rows = time.perf_counter() - t0
            est = t_deq * w.E + t_rows / rows * w.R
            result["cpu_baseline"] = {"value": w.T / est, "unit": "tokens/s", "cores": oracle.num_threads(),
                                      "kind": "oracle",
                                      "sample": "expert FFN on %d rows of expert 0 (%.1f s) + dequantising one expert (%.1f s), scaled to %d rows and %d experts"
                                                % (rows, t_rows, t_deq, w.R, w.E)}
    del layer, ring, x, masters
    gc.collect()
    torch.cuda.empty_cache()
    return result


def main():
    args = parse()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives); use --gpus 1")

    import torch

    from paper_2211_10017_amd import binding

    binding.load()                       # fails loudly if the HIP library is not built
    head = measure(args.workload, args, not args.no_cpu_baseline, True)
    result = {
        "metric": "MoE expert-layer tokens/sec", "value": head["value"], "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": head["dtype"],
        "data": "synthetic", "config": head["config"], "roofline": head["roofline"], "step_us": head["step_us"],
        "box_peaks": box_peaks(torch, binding),
    }
    if "cpu_baseline" in head:
        result["cpu_baseline"] = head["cpu_baseline"]
    # the other configurations, same protocol and the same --steps / --warmup, each with its own
    # roofline block (the headline fields above stay those of the first workload)
    if not args.no_others and args.workload == "c2" and args.finished == 0:
        others = {}
        for name in OTHERS:
            r = measure(name, args, (not args.no_cpu_baseline) and name == "c1", False)
            others[name] = r
        result["other_workloads"] = others
    print(json.dumps(result))


if __name__ == "__main__":
    main()
