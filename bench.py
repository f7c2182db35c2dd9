#!/usr/bin/env python3
"""Benchmark of the MoE expert FFN layer on one MI355X.

A step is one pass of the whole hot path (gate -> permute -> grouped FFN -> combine) over one
batch of seeded synthetic tokens, with inputs and quantised weights already resident in HBM.
Prints ONE JSON line: whole-job tokens/s, the roofline figures of the dominant kernel (the
grouped weight-quantised GEMM) from HIP events, and the CPU oracle timed beside it.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2] [--no-cpu-baseline]

Cold-cache protocol: the weights of the small workloads would fit in the 256 MB last-level
cache, so the layer cycles through a ring of identical weight copies (>= 1 GiB in total), one
copy per step; every step therefore streams its weights from HBM.
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

# HBM bytes per launch of the grouped GEMM, from `rocprofv3 --pmc FETCH_SIZE` and `--pmc WRITE_SIZE`
# runs of this file (profiles/stream_unrolled_c2_traffic.md, profiles/grouped_gemm_c5_counters.md): counter readings scaled by what the same
# counters read for a plain 256 MiB device copy (FETCH_SIZE x 2.0, WRITE_SIZE x 1.0).
MEASURED_TRAFFIC_BYTES_PER_LAUNCH = {"c2": 71.1e6, "c5": 4.30e9}

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_F16_PEAK_TFLOPS = 2500.0  # MI355X dense fp16 MFMA


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2")
    ap.add_argument("--no-cpu-baseline", action="store_true")
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


def main():
    args = parse()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives); use --gpus 1")

    import numpy as np
    import torch

    from paper_2211_10017_amd import MoEExpertLayer, binding
    from paper_2211_10017_amd import workloads as W

    binding.load()                       # fails loudly if the HIP library is not built
    w = W.WORKLOADS[args.workload]
    dev = "cuda:0"
    tdt = torch.float16 if w.act == "f16" else torch.bfloat16
    layer = MoEExpertLayer(w.T, w.d, w.F, w.E, w.k, w.bits, w.group_size, act_dtype=tdt,
                           renormalize=w.renormalize, device=dev)
    x_np, wg_np, bias_np = W.activations(w), W.gate_weight(w), W.gate_bias(w)
    layer.wg.copy_(torch.from_numpy(wg_np).to(dev, tdt))
    if bias_np is not None:
        layer.gate_bias = torch.from_numpy(bias_np).to(dev)
    x = torch.from_numpy(x_np).to(dev, tdt)
    keep_masters = (not args.no_cpu_baseline) and w.E * w.d * w.F * 8 <= 4e9
    masters = {1: [], 2: []}
    for which in (1, 2):
        for e0, ms in W.expert_weight_batches(w, which):
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

    for i in range(ncopy):                # first use of every ring copy marshals its argument lists: not a step
        step(i)
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    tokens_per_s = w.T * args.steps / elapsed

    # ---- the same K steps again with HIP events around the grouped-GEMM launches (events are on
    # torch's current stream, which is the stream the library launches on)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for i in range(args.steps):
        layer.w1_packed, layer.s1, layer.w2_packed, layer.s2 = ring[i % ncopy]
        layer.gate(x, finished)
        layer.permute(x, finished)
        ev[i][0].record()
        layer.ffn(x, finished)
        ev[i][1].record()
        layer.combine(x, finished)
    torch.cuda.synchronize()
    ffn_ms = np.array([a.elapsed_time(b) for a, b in ev])
    launches_per_ffn = 2                       # fc1 and fc2 are two launches of the same kernel
    launch_s = float(ffn_ms.mean()) * 1e-3 / launches_per_ffn

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
    roofline["traffic"] = MEASURED_TRAFFIC_BYTES_PER_LAUNCH.get(w.name) if args.finished == 0 else None
    # which GEMM kernel the library's dispatch rule picks for these sizes (bf16 rows and everything the
    # routing-fused entry point takes run in the LDS-tiled kernel, the rest streams)
    tiled = w.act == "bf16" or binding.moe_grouped_ffn_wq_routed_supported(w.R, w.E, w.T, w.d, w.F, w.bits, w.group_size, torch.float16)
    roofline.update({"kernel": "grouped_gemm_kernel" if tiled else "stream_unrolled_kernel", "launches_per_step": launches_per_ffn,
                     "avg_launch_us": launch_s * 1e6, "ffn_us_median": float(np.median(ffn_ms)) * 1e3,
                     "ffn_us_min": float(ffn_ms.min()) * 1e3, "active_experts": active,
                     "algorithmic_bytes_per_step": int(bytes_ffn), "flops_per_step": flops_ffn,
                     "weight_ring_copies": ncopy})

    result = {
        "metric": "MoE expert-layer tokens/sec", "value": tokens_per_s, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.act,
        "data": "synthetic", "config": {"workload": describe(w), "weights": "int%d" % w.bits,
                                        "routed_rows": w.R, "cold_weights": ncopy > 1,
                                        **({"finished_fraction": args.finished, "active_rows": active_rows}
                                           if args.finished > 0 else {})},
        "roofline": roofline,
    }

    # ---- the CPU oracle on the same inputs, on this machine's host cores (a reported baseline)
    if not args.no_cpu_baseline:
        import oracle
        act = oracle.F16 if w.act == "f16" else oracle.BF16
        if keep_masters:
            q1, s1 = oracle.quantize(np.stack(masters[1]), w.bits, w.group_size)
            q2, s2 = oracle.quantize(np.stack(masters[2]), w.bits, w.group_size)
            reps, spent = 0, 0.0
            while spent < 10.0 and reps < 50:
                t0 = time.perf_counter()
                oracle.moe_layer(x_np, wg_np, bias_np, q1, s1, q2, s2, w.k, w.group_size, act,
                                 renormalize=w.renormalize)
                spent += time.perf_counter() - t0
                reps += 1
            result["cpu_baseline"] = {"value": w.T * reps / spent, "unit": "tokens/s",
                                      "cores": oracle.num_threads(), "kind": "oracle",
                                      "sample": "%d full passes of the same layer (all %d tokens), %.1f s" % (reps, w.T, spent)}
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
    print(json.dumps(result))


if __name__ == "__main__":
    main()
