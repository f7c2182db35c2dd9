"""Throughput of the vendor library's plain FP16 GEMM (torch.matmul -> hipBLASLt) on the shapes of
workload c5's two matrix products, with normally distributed and with all-zero operands.  A
reference point for the MFMA roofline fraction bench.py reports: the same chip, the same shapes,
no dequantisation and no grouping.  Not used by the library."""
import torch


def main():
    dev = "cuda:0"
    for (m, k, n) in [(16384, 4096, 16384), (16384, 16384, 4096)]:
        a = torch.randn(m, k, device=dev, dtype=torch.float16)
        b = torch.randn(k, n, device=dev, dtype=torch.float16)
        for label in ("N(0,1)", "zero"):
            if label == "zero":
                a.zero_()
                b.zero_()
            for _ in range(3):
                a @ b
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(10):
                a @ b
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / 10
            print("library fp16 gemm %dx%dx%d, %s operands: %.3f ms, %.0f TFLOP/s" % (m, k, n, label, ms, 2.0 * m * k * n / ms / 1e9), flush=True)


if __name__ == "__main__":
    main()
