"""The tiled grouped GEMM sends its activation rows (fp16, or bf16 converted to scaled fp16 beforehand) from global memory straight into LDS and waits for
them with a hand-counted `s_waitcnt vmcnt(n)`, n = the weight loads issued after them.  The library is
built a second time (libmoe_wq_waitall.so) with every such wait replaced by a wait for ALL loads, which
needs no counting.  If a compiler change ever merged, split or reordered one of the counted loads, the
normal build would read stale rows; this test runs every direct-to-LDS variant of the kernel in both
builds and compares the outputs bit for bit."""
import ctypes
import os

import numpy as np
import pytest
import torch

from helpers import to_dev
from paper_2211_10017_amd import binding as B

pytestmark = pytest.mark.gpu
WAITALL = os.path.join(os.path.dirname(B.LIB_PATH), "libmoe_wq_waitall.so")


def _ffn(lib, x, off, R, E, d, F, bits, g, p1, s1, p2, s2, y_dtype):
    vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    lib.moe_grouped_ffn_wq.restype = i
    lib.moe_grouped_ffn_wq.argtypes = [vp, i, vp, i, i, i, i, i, i, i, i, vp, vp, vp, vp, vp, vp, vp, i, vp, sz, vp]
    lib.moe_last_ffn_kernels.restype = ctypes.c_char_p
    y = torch.full((R, d), float("nan"), dtype=y_dtype, device=x.device)
    ws = torch.empty(B.moe_grouped_ffn_wq_workspace_bytes(R, d, F, E, x.dtype), dtype=torch.uint8, device=x.device)
    rc = lib.moe_grouped_ffn_wq(x.data_ptr(), B._DT[x.dtype], off.data_ptr(), R, E, 0, d, F, bits, g, 0, p1.data_ptr(), s1.data_ptr(), None,
                                p2.data_ptr(), s2.data_ptr(), None, y.data_ptr(), B._DT[y_dtype], ws.data_ptr(), ws.numel(),
                                torch.cuda.current_stream().cuda_stream)
    assert rc == 0
    torch.cuda.synchronize()
    return y, lib.moe_last_ffn_kernels().decode()


@pytest.mark.parametrize("rows,d,F,bits,g,y_dt,x_dt", [(*c, torch.float16) for c in [
    ([20, 31, 5, 0, 17], 192, 256, 4, 0, torch.float16),            # 32-row tiles; 3 and 4 K steps (odd, even)
    ([20, 31, 5, 0, 17], 192, 256, 8, 64, torch.float32),
    ([60, 50, 33, 5], 192, 320, 4, 64, torch.float32),              # 64-row tiles, last tiles with one live row tile; 3 and 5 K steps
    ([60, 50, 33, 5], 256, 128, 8, 0, torch.float16),               # 4 and 2 K steps
    ([270, 257, 130, 20], 2112, 2176, 4, 0, torch.float16),         # 128-row tiles (3, 3, 2 + 1 and 1 live row tiles); 33 and 34 K steps
    ([270, 257, 130, 20], 2112, 2176, 4, 64, torch.float32),        # ... with a scale per group
    ([300, 290, 270], 2112, 2112, 8, 0, torch.float16),             # tallest 8-bit tiles: weights fetched one step ahead
    ([300, 290, 270], 2112, 2112, 8, 64, torch.float32)]] + [
    # bf16 rows: fc1 keeps the group scales out of the weights (group sums folded in fp32 for groups of 128, two-term weights otherwise)
    ([20, 31, 5, 0, 17], 256, 384, 4, 128, torch.float32, torch.bfloat16),      # 32-row tiles, group sums
    ([60, 50, 33, 5], 384, 256, 8, 128, torch.float32, torch.bfloat16),         # 64-row tiles, group sums
    ([270, 257, 130, 20], 2176, 2304, 4, 128, torch.float32, torch.bfloat16),   # taller experts: group sums stay on 64-row tiles
    ([60, 50, 33, 5], 192, 320, 4, 64, torch.float32, torch.bfloat16),          # two-term weights, 64-row tiles
    ([270, 257, 130, 20], 2112, 2176, 8, 64, torch.float32, torch.bfloat16)])   # two-term weights, 128-row tiles
def test_counted_waits_equal_waiting_for_all_loads(rows, d, F, bits, g, y_dt, x_dt):
    print(f"wait guard rows={rows} d={d} F={F} bits={bits} g={g} y={y_dt} x={x_dt}", flush=True)
    assert os.path.exists(WAITALL), "libmoe_wq_waitall.so is built by paper_2211_10017_amd.build together with the library"
    rng = np.random.default_rng(sum(rows) + d + bits + g)
    E = len(rows)
    off = to_dev(np.concatenate([[0], np.cumsum(rows)]).astype(np.int32), torch.int32)
    R = int(sum(rows))
    x = to_dev(rng.standard_normal((R, d)).astype(np.float32), x_dt)
    w1 = to_dev((rng.standard_normal((E, d, F)) * 0.05).astype(np.float32), torch.float32)
    w2 = to_dev((rng.standard_normal((E, F, d)) * 0.05).astype(np.float32), torch.float32)
    _, s1, p1 = B.moe_quantize_experts(w1, bits, g, want_canon=False)
    _, s2, p2 = B.moe_quantize_experts(w2, bits, g, want_canon=False)
    plain, kernels = _ffn(B.load(), x, off, R, E, d, F, bits, g, p1, s1, p2, s2, y_dt)
    other, kernels2 = _ffn(ctypes.CDLL(WAITALL), x, off, R, E, d, F, bits, g, p1, s1, p2, s2, y_dt)
    assert kernels == kernels2 == "grouped_gemm_kernel grouped_gemm_kernel"      # both GEMMs in the tiled kernel
    assert torch.isfinite(plain.float()).all()
    assert torch.equal(plain, other)
