#!/usr/bin/env python3
"""The experiment of Table 1 (Sec. 4.1) on one MI355X: time of ONE grouped GEMM, A [m x 1024] per
active expert against B [1024 x 4096], about 40 tokens spread evenly over 1, 4, 8, 16, 24 or 32
active experts of 32, with fp16, int8 and int4 weights, normalised to the fp16-weight kernel of
this library; plus the same int8 / int4 kernels with the chip's integer-to-float instructions
instead of the magic-number conversion (Sec. 3.4.1).  Weights come from a ring of copies (more than the
256 MB last-level cache), so every launch streams them from HBM.  Prints a markdown table.

    python -m paper_2211_10017_amd.table1_sweep [--tokens 40] [--iters 100]
"""
from __future__ import annotations

import argparse

import numpy as np
import torch

from . import binding as B

K, N, E = 1024, 4096, 32


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--tokens", type=int, default=40)
    ap.add_argument("--iters", type=int, default=200)
    args = ap.parse_args()
    dev = "cuda:0"
    B.load()
    rng = np.random.Generator(np.random.Philox(key=[7, 0]))
    w = torch.from_numpy((rng.standard_normal((E, K, N)) * 0.02).astype(np.float32)).to(dev)
    variants = {}
    variants["fp16"] = (16, False, B.moe_pack_fp16_experts(w), None)
    for bits in (8, 4):
        _, s, p = B.moe_quantize_experts(w, bits, 0, want_canon=False)
        variants["int%d" % bits] = (bits, False, p, s)
        variants["int%d native I2F" % bits] = (bits, True, p, s)
    del w
    ring = {}
    for name, (bits, native, p, s) in variants.items():
        copies = max(2, int(-(-(1 << 30) // p.numel())))
        ring[name] = [p] + [p.clone() for _ in range(min(copies, 16) - 1)]
    x_all = torch.from_numpy(rng.standard_normal((args.tokens, K)).astype(np.float32)).to(dev, torch.float16)
    y = torch.empty((args.tokens, N), dtype=torch.float16, device=dev)
    print("| active experts | rows per expert | " + " | ".join("%s us" % n for n in variants) +
          " | int8 / fp16 | int4 / fp16 | int4 GB/s |")
    print("|---|---|" + "---|" * (len(variants) + 3))
    for active in (1, 4, 8, 16, 24, 32):
        rows = np.zeros(E, dtype=np.int64)
        rows[:active] = args.tokens // active
        rows[: args.tokens % active] += 1
        off = torch.from_numpy(np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)).to(dev)
        bound = int(rows.max())
        times = {}
        for name, (bits, native, p, s) in variants.items():
            bufs = ring[name]

            def call(i):
                B.moe_grouped_gemm_wq(x_all, off, E, K, N, bits, bufs[i % len(bufs)], s, native_convert=native, y=y,
                                      max_rows_per_expert=bound)
            for i in range(5):
                call(i)
            torch.cuda.synchronize()
            # events around batches of launches, so that the queue never runs dry while the host
            # prepares the next call
            batch, nb = 10, max(1, args.iters // 10)
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(nb)]
            for j in range(nb):
                ev[j][0].record()
                for i in range(batch):
                    call(j * batch + i)
                ev[j][1].record()
            torch.cuda.synchronize()
            times[name] = float(np.median([a.elapsed_time(b) for a, b in ev])) * 1e3 / batch
        gbs = active * K * N / 2 / times["int4"] / 1e3
        print("| %d | %s | " % (active, "%d" % rows[0] if rows[0] == rows[active - 1] else "%d-%d" % (rows[active - 1], rows[0])) +
              " | ".join("%.1f" % times[n] for n in variants) +
              " | %.2fx | %.2fx | %.0f |" % (times["fp16"] / times["int8"], times["fp16"] / times["int4"], gbs), flush=True)


if __name__ == "__main__":
    main()
