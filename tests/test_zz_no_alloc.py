"""GPU test of moe_grouped_ffn_wq_noalloc, the entry point for callers that cannot allocate: its
output must equal moe_grouped_ffn_wq's (the same kernels run, so bit for bit, which is well inside
the layer's tolerance against the oracle) on two calls in a row, the second with a smaller input
that leaves most of the first call's h behind in the built-in scratch array."""
import numpy as np
import pytest
import torch

import oracle
from helpers import MAX_ABS_TOL, REL_L2_TOL, error_metrics, to_dev
from paper_2211_10017_amd import binding as B

pytestmark = pytest.mark.gpu


def _case(rows, d, F, bits, g, seed):
    rng = np.random.default_rng(seed)
    E = len(rows)
    off = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    R = int(off[-1])
    x = rng.standard_normal((R, d)).astype(np.float16).astype(np.float32)
    w1 = (rng.standard_normal((E, d, F)) * 0.05).astype(np.float32)
    w2 = (rng.standard_normal((E, F, d)) * 0.05).astype(np.float32)
    _, s1, p1 = B.moe_quantize_experts(to_dev(w1, torch.float32), bits, g, want_canon=False)
    _, s2, p2 = B.moe_quantize_experts(to_dev(w2, torch.float32), bits, g, want_canon=False)
    q1, os1 = oracle.quantize(w1, bits, g)
    q2, os2 = oracle.quantize(w2, bits, g)
    want = oracle.grouped_ffn(x, off, q1, os1, q2, os2, g, oracle.F16)
    return dict(E=E, d=d, F=F, bits=bits, g=g, x=to_dev(x, torch.float16), off=to_dev(off, torch.int32),
                p1=p1, s1=s1, p2=p2, s2=s2, want=want, R=R)


def _run_both(c):
    print(f"no-alloc ffn R={c['R']} d={c['d']} F={c['F']} bits={c['bits']} g={c['g']}", flush=True)
    y_ws = B.moe_grouped_ffn_wq(c["x"], c["off"], c["E"], c["d"], c["F"], c["bits"], c["g"], c["p1"], c["s1"], c["p2"],
                                c["s2"], y_dtype=torch.float32)
    y_na = torch.full((c["R"], c["d"]), float("nan"), dtype=torch.float32, device=c["x"].device)
    B.moe_grouped_ffn_wq_noalloc(c["x"], c["off"], c["E"], c["d"], c["F"], c["bits"], c["g"], c["p1"], c["s1"], c["p2"],
                                 c["s2"], y_na)
    torch.cuda.synchronize()
    assert torch.equal(y_na, y_ws)                                     # the same kernels: bit for bit
    max_abs, rel = error_metrics(y_na.cpu().numpy(), c["want"])      # and so within the oracle's tolerance
    print(f"   max_abs={max_abs:.3e} rel_l2={rel:.3e}", flush=True)
    assert max_abs <= MAX_ABS_TOL and rel <= REL_L2_TOL


def test_noalloc_ffn_equals_the_workspace_entry_point_on_two_calls_in_a_row():
    assert B.load().moe_grouped_ffn_wq_noalloc_max_bytes() == 8 << 20
    big = _case([5, 0, 33, 1, 70, 9], 256, 1024, 4, 0, seed=21)       # tiled kernel, 118 rows of F = 1024
    small = _case([3, 4, 0, 2], 1024, 2048, 4, 0, seed=22)            # decode-sized: the streaming kernels, 9 rows
    _run_both(big)
    _run_both(small)                                                   # h of the first call is still in the array
    _run_both(big)


def test_noalloc_ffn_refuses_what_does_not_fit():
    c = _case([2], 64, 64, 4, 0, seed=23)
    lib = B.load()
    vp = lambda t: None if t is None else t.data_ptr()  # noqa: E731
    y = torch.empty((4096, 64), dtype=torch.float16, device="cuda:0")
    # 4096 rows of F = 2048 would need 16 MiB of h: refused before any launch
    rc = lib.moe_grouped_ffn_wq_noalloc(vp(c["x"]), 0, vp(c["off"]), 4096, 1, 0, 64, 2048, 4, 0, 0, vp(c["p1"]), vp(c["s1"]), None,
                                        vp(c["p2"]), vp(c["s2"]), None, vp(y), 0, None)
    assert rc == 3 and b"scratch" in lib.moe_last_error()
