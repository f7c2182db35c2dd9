"""GPU parity, step by step, through the C-ABI: each entry point against the oracle on small
seeded inputs that still span several tiles, ragged tails and the degenerate cases."""
import numpy as np
import pytest
import torch

import oracle
from helpers import MAX_ABS_TOL, REL_L2_TOL, error_metrics, oracle_dtype_code, to_dev
from paper_2211_10017_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _say(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------ quantise
@pytest.mark.parametrize("bits,g,E,K,N", [(8, 0, 3, 128, 96), (4, 0, 2, 192, 64), (4, 64, 2, 256, 160),
                                          (8, 128, 1, 256, 32), (4, 128, 5, 1024, 224)])
def test_quantize_bit_exact(bits, g, E, K, N):
    _say(f"quantize bits={bits} g={g} E={E} K={K} N={N}")
    rng = np.random.default_rng(bits + g + N)
    w = (rng.standard_normal((E, K, N)) * 0.02).astype(np.float32)
    w[0, :, 3] = 0.0                                            # dead channel
    w[E - 1, 5, 7] = 0.3                                        # an outlier that sets a scale
    # exact ties: make some weights exactly 2.5 steps of a power-of-two scale
    w[0, :, 1] = 0.0
    w[0, 0, 1] = (2 ** (bits - 1) - 1) * 2.0 ** -6
    w[0, 1, 1] = 2.5 * 2.0 ** -6
    w[0, 2, 1] = -3.5 * 2.0 ** -6
    oq, os_ = oracle.quantize(w, bits, g)
    q_canon, scales, q_packed = B.moe_quantize_experts(to_dev(w, torch.float32), bits, g)
    torch.cuda.synchronize()
    want = oq if bits == 8 else oracle.pack_int4(oq)
    assert np.array_equal(q_canon.cpu().numpy().view(want.dtype), want)
    assert np.array_equal(scales.cpu().numpy().view(np.uint16), os_)
    assert q_packed.numel() == E * K * N * bits // 8
    # one expert at a time gives the same bytes as one call over all experts
    if E > 1:
        qc1, sc1, qp1 = B.moe_quantize_experts(to_dev(w[1:2], torch.float32), bits, g)
        nb = K * N * bits // 8
        assert torch.equal(qp1, q_packed[nb:2 * nb]) and torch.equal(sc1[0], scales[1])


# ------------------------------------------------------------------ gate
@pytest.mark.parametrize("T,d,E,k,act", [
    (64, 1024, 32, 2, "f16"), (37, 64, 1, 1, "f16"), (130, 192, 3, 2, "f16"), (256, 512, 8, 1, "f16"),
    (100, 640, 64, 2, "bf16"), (77, 2048, 128, 2, "f16"), (33, 256, 100, 1, "bf16"), (19, 128, 200, 2, "f16"),
    (5, 4096, 64, 2, "f16"), (4133, 256, 64, 2, "f16"), (4100, 128, 130, 1, "bf16"), (4133, 264, 64, 2, "bf16"),
    # a token per lane (many tokens, 64 experts): ragged last block; one, three and six feature blocks
    (16400, 256, 64, 2, "f16"), (16384, 128, 64, 1, "f16"), (16501, 384, 64, 2, "f16"), (17000, 768, 64, 1, "f16"),
    # bf16, 64 experts: thirty-two tokens per lane from 8192 tokens on
    (8200, 256, 64, 2, "bf16"), (8229, 136, 64, 1, "bf16")])
def test_gate_routing_bit_exact(T, d, E, k, act):
    _say(f"gate T={T} d={d} E={E} k={k} {act}")
    rng = np.random.default_rng(T + d + E)
    tdt = torch.float16 if act == "f16" else torch.bfloat16
    x = to_dev(rng.standard_normal((T, d)).astype(np.float32), tdt)
    wg = to_dev((rng.standard_normal((d, E)) * 0.02).astype(np.float32), tdt)
    bias = rng.uniform(-0.2, 0.2, E).astype(np.float32) if E % 2 == 0 else None
    for renorm in (True, False):
        oi, osc = oracle.gate(x.float().cpu().numpy(), wg.float().cpu().numpy(), bias, k, renorm)
        gi, gs = B.moe_gate_topk(x, wg, None if bias is None else to_dev(bias, torch.float32), k, renorm)
        torch.cuda.synchronize()
        assert np.array_equal(gi.cpu().numpy(), oi)
        assert np.allclose(gs.cpu().numpy(), osc, rtol=1e-5, atol=1e-9)


def test_gate_ties_and_equal_logits():
    _say("gate ties")
    x = torch.ones((9, 64), dtype=torch.float16, device=DEV)
    wg = torch.zeros((64, 6), dtype=torch.float16, device=DEV)
    gi, gs = B.moe_gate_topk(x, wg, None, 2, True)
    assert np.array_equal(gi.cpu().numpy(), np.tile([0, 1], (9, 1))) and np.allclose(gs.cpu().numpy(), 0.5)
    wg[0, 2] = 1.0
    wg[0, 5] = 1.0
    gi, _ = B.moe_gate_topk(x, wg, None, 2, True)
    assert np.array_equal(gi.cpu().numpy(), np.tile([2, 5], (9, 1)))
    gi, gs = B.moe_gate_topk(x[:0], wg, None, 1, True)           # T = 0 is a no-op
    assert gi.shape == (0, 1)
    # the same with a token per lane (many tokens, 64 experts)
    x = torch.ones((16389, 128), dtype=torch.float16, device=DEV)
    wg = torch.zeros((128, 64), dtype=torch.float16, device=DEV)
    gi, gs = B.moe_gate_topk(x, wg, None, 2, True)
    assert np.array_equal(gi.cpu().numpy(), np.tile([0, 1], (16389, 1))) and np.allclose(gs.cpu().numpy(), 0.5)
    wg[0, 7] = 1.0
    wg[0, 63] = 1.0
    gi, _ = B.moe_gate_topk(x, wg, None, 2, True)
    assert np.array_equal(gi.cpu().numpy(), np.tile([7, 63], (16389, 1)))
    gi, gs = B.moe_gate_topk(x, wg, None, 1, True)
    assert (gi.cpu().numpy() == 7).all()


# ------------------------------------------------------------------ permute
@pytest.mark.parametrize("T,k,E,d", [(64, 2, 32, 1024), (1, 1, 4, 64), (300, 2, 13, 128), (4096, 1, 64, 64),
                                      (5000, 2, 128, 64), (16384, 1, 64, 256), (4500, 1, 1, 64), (700, 2, 200, 72)])
def test_permute_bit_exact(T, k, E, d):
    _say(f"permute T={T} k={k} E={E} d={d}")
    rng = np.random.default_rng(T + E)
    hi = max(1, E - 2) if E > 4 else E                          # leave the last experts empty
    idx = rng.integers(0, hi, size=(T, k)).astype(np.int32)
    if E > 8:
        idx[idx == 3] = 4                                        # an empty expert in the middle
    x = rng.standard_normal((T, d)).astype(np.float16)
    perm_src, inv_perm, off = oracle.permute(idx, E)
    xp, ps, ip, of = B.moe_permute(to_dev(idx, torch.int32), to_dev(x, torch.float16), E)
    torch.cuda.synchronize()
    assert np.array_equal(of.cpu().numpy(), off)
    assert np.array_equal(ps.cpu().numpy(), perm_src)
    assert np.array_equal(ip.cpu().numpy(), inv_perm)
    assert np.array_equal(xp.cpu().numpy(), x[perm_src // k])


def test_permute_no_tokens():
    _say("permute T=0")
    idx = torch.empty((0, 2), dtype=torch.int32, device=DEV)
    x = torch.empty((0, 64), dtype=torch.float16, device=DEV)
    xp, ps, ip, of = B.moe_permute(idx, x, 5)
    torch.cuda.synchronize()
    assert xp.shape == (0, 64) and not of.cpu().numpy().any() and of.numel() == 6


# ------------------------------------------------------------------ grouped FFN
def _ffn_case(rows_per_expert, d, F, bits, g, act, y_dt, seed, with_bias=False, activation="relu", bound=0):
    rng = np.random.default_rng(seed)
    E = len(rows_per_expert)
    off = np.concatenate([[0], np.cumsum(rows_per_expert)]).astype(np.int32)
    R = int(off[-1])
    tdt = torch.float16 if act == "f16" else torch.bfloat16
    x = to_dev(rng.standard_normal((R, d)).astype(np.float32), tdt)
    w1 = (rng.standard_normal((E, d, F)) * 0.05).astype(np.float32)
    w2 = (rng.standard_normal((E, F, d)) * 0.05).astype(np.float32)
    _, s1, p1 = B.moe_quantize_experts(to_dev(w1, torch.float32), bits, g, want_canon=False)
    _, s2, p2 = B.moe_quantize_experts(to_dev(w2, torch.float32), bits, g, want_canon=False)
    q1, os1 = oracle.quantize(w1, bits, g)
    q2, os2 = oracle.quantize(w2, bits, g)
    assert np.array_equal(s1.cpu().numpy().view(np.uint16), os1)
    b1 = b2 = ob1 = ob2 = None
    if with_bias:
        ob1 = rng.standard_normal((E, F)).astype(np.float16).astype(np.float32) * 0.1
        ob2 = rng.standard_normal((E, d)).astype(np.float16).astype(np.float32) * 0.1
        b1, b2 = to_dev(ob1, torch.float16), to_dev(ob2, torch.float16)
    y = B.moe_grouped_ffn_wq(x, to_dev(off, torch.int32), E, d, F, bits, g, p1, s1, p2, s2, b1, b2, y_dtype=y_dt,
                             activation=activation, max_rows_per_expert=bound)
    torch.cuda.synchronize()
    want = oracle.grouped_ffn(x.float().cpu().numpy(), off, q1, os1, q2, os2, g, oracle_dtype_code(tdt), ob1, ob2,
                              activation=B.ACTIVATIONS[activation])
    want = oracle.round_to(want, oracle_dtype_code(y_dt))
    return y.float().cpu().numpy(), want


@pytest.mark.parametrize("rows,d,F,bits,g,act,y_dt", [
    ([5, 0, 33, 1, 70], 128, 256, 4, 0, "f16", torch.float16),
    ([40], 1024, 4096, 4, 0, "f16", torch.float16),
    ([4], 1024, 4096, 4, 0, "f16", torch.float16),
    ([8, 9], 1024, 2048, 4, 0, "f16", torch.float32),
    ([32, 33, 1], 1024, 1024, 4, 0, "f16", torch.float32),
    ([7, 0, 16], 512, 2048, 8, 0, "f16", torch.float16),
    ([3, 4, 0, 0, 9, 2, 1, 6], 1024, 4096, 4, 0, "f16", torch.float32),
    ([20, 0, 17, 5], 1024, 3072, 4, 0, "f16", torch.float16),
    ([6, 11], 1536, 512, 8, 0, "f16", torch.float32),
    ([3, 0, 12], 1024, 2048, 8, 0, "f16", torch.float16),
    ([31, 32, 33, 64, 65, 0, 129], 192, 320, 8, 0, "f16", torch.float16),
    ([100, 260, 7], 256, 512, 4, 128, "f16", torch.float16),
    ([17, 140], 512, 256, 8, 64, "f16", torch.float32),
    ([9, 200, 0, 45], 256, 512, 4, 128, "bf16", torch.float32),
    ([64, 3], 128, 192, 8, 0, "bf16", torch.float32),
    ([150, 20], 256, 256, 4, 64, "bf16", torch.float32),
    ([300, 70, 129], 256, 320, 8, 0, "f16", torch.float16),        # tallest 8-bit tiles (weights fetched one step ahead), rows dealt 96+96+96+12
    ([290, 131], 128, 192, 8, 0, "bf16", torch.float32),
    ([270, 257, 1], 192, 256, 4, 0, "f16", torch.float32),          # balanced row tiles: 96+96+78 and 96+96+65
    ([2, 11, 5], 256, 2048, 8, 0, "f16", torch.float16),            # fc2 splits K over the wavefronts, two channel tiles per block
    # K above 2048 and many rows per expert: the 128-row tiles (shorter K loops and 8-bit weights up to 256 rows run 64-row tiles)
    ([270, 257, 1], 2112, 2176, 4, 0, "f16", torch.float32),
    ([300, 270, 259], 2112, 2176, 8, 0, "f16", torch.float16),      # tallest 8-bit tiles: weights fetched one step ahead
    ([300, 280], 2112, 2176, 8, 64, "f16", torch.float32),
    ([290, 300], 2112, 2112, 8, 0, "bf16", torch.float32),
    ([150, 120], 2112, 2112, 4, 64, "bf16", torch.float32),         # two-term group scales in 128-row tiles
    # 4-bit weights, group scales, fp16 rows, K above 2048 in both GEMMs, more than 64 rows per expert on
    # average: the 128-row tiles with a scale per group (the variant the largest workload's fp16 pass runs),
    # every row compared; rows dealt 96+96+78, 96+96+65 and 96+34
    ([270, 257, 130], 2112, 2176, 4, 64, "f16", torch.float16),
    ([270, 257, 130], 2176, 2304, 4, 128, "f16", torch.float32),
    ([129, 288, 1, 256], 2304, 2176, 4, 128, "f16", torch.float16), # 128 + 1 rows; nine 32-row units in three tiles; one row; two full tiles
])
def test_grouped_ffn_matches_oracle(rows, d, F, bits, g, act, y_dt):
    _say(f"ffn rows={rows} d={d} F={F} bits={bits} g={g} {act} y={y_dt}")
    got, want = _ffn_case(rows, d, F, bits, g, act, y_dt, seed=sum(rows) + d + bits)
    max_abs, rel = error_metrics(got, want)
    _say(f"   max_abs={max_abs:.3e} rel_l2={rel:.3e}")
    assert max_abs <= MAX_ABS_TOL and rel <= REL_L2_TOL


@pytest.mark.parametrize("bits,g", [(4, 128), (8, 0), (4, 64)])
def test_grouped_ffn_bf16_rows_of_any_magnitude(bits, g):
    """bf16 rows far outside the FP16 range (rows scaled by 2^-40 ... 2^40) and with elements down to 2^-30 of their
    row's largest: every row goes into the GEMMs scaled by its own power of two and comes out scaled back.  Without
    biases the layer is homogeneous in a row's scale, so each row is compared relative to its own size."""
    _say(f"ffn bf16 rows of any magnitude bits={bits} g={g}")
    rng = np.random.default_rng(11 + bits + g)
    rows, d, F = [40, 100], 256, 256
    E, R = len(rows), sum(rows)
    off = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    row_scale = 2.0 ** (8 * (np.arange(R) % 11 - 5))
    col_scale = 2.0 ** (-2.0 * (np.arange(d) % 16))
    x = to_dev((rng.standard_normal((R, d)) * row_scale[:, None] * col_scale[None, :]).astype(np.float32), torch.bfloat16)
    w1 = (rng.standard_normal((E, d, F)) * 0.05).astype(np.float32)
    w2 = (rng.standard_normal((E, F, d)) * 0.05).astype(np.float32)
    _, s1, p1 = B.moe_quantize_experts(to_dev(w1, torch.float32), bits, g, want_canon=False)
    _, s2, p2 = B.moe_quantize_experts(to_dev(w2, torch.float32), bits, g, want_canon=False)
    q1, os1 = oracle.quantize(w1, bits, g)
    q2, os2 = oracle.quantize(w2, bits, g)
    y = B.moe_grouped_ffn_wq(x, to_dev(off, torch.int32), E, d, F, bits, g, p1, s1, p2, s2, y_dtype=torch.float32)
    torch.cuda.synchronize()
    got = y.cpu().numpy().astype(np.float64)
    want = oracle.grouped_ffn(x.float().cpu().numpy(), off, q1, os1, q2, os2, g, oracle.BF16).astype(np.float64)
    assert np.isfinite(got).all()
    size = np.sqrt((want ** 2).sum(axis=1))
    assert (size > 0).all() and size.max() / size.min() > 2.0 ** 70          # the rows really span the range
    rel = np.sqrt(((got - want) ** 2).sum(axis=1)) / size
    _say(f"   row sizes 2^{np.log2(size.min()):.0f} .. 2^{np.log2(size.max()):.0f}; worst relative L2 error of a row {rel.max():.3e}")
    assert rel.max() <= 2 * REL_L2_TOL


@pytest.mark.parametrize("rows,d,F,bits", [
    # a row bound of at most 64, but several row groups per expert and enough row tiles to fill the chip: the tiled kernel
    ([40, 37, 44, 40, 1, 40, 39, 40, 64, 40, 33, 40], 1024, 4096, 4),
    # fc1 in row tiles, fc2 (two column blocks: too few tiles) in the run-loop streaming kernel
    ([20] * 14, 512, 2560, 8),
    # decode-sized: both GEMMs stream whatever the rows per expert
    ([60, 64, 3], 1024, 4096, 4),
])
def test_grouped_ffn_with_a_row_bound_matches_oracle(rows, d, F, bits):
    _say(f"ffn with row bound rows={rows} d={d} F={F} bits={bits}")
    got, want = _ffn_case(rows, d, F, bits, 0, "f16", torch.float32, seed=sum(rows) + bits, bound=max(rows))
    max_abs, rel = error_metrics(got, want)
    _say(f"   max_abs={max_abs:.3e} rel_l2={rel:.3e}")
    assert max_abs <= MAX_ABS_TOL and rel <= REL_L2_TOL


def test_grouped_ffn_biases():
    _say("ffn with biases")
    got, want = _ffn_case([20, 45, 3], 128, 256, 8, 0, "f16", torch.float32, seed=5, with_bias=True)
    max_abs, rel = error_metrics(got, want)
    assert max_abs <= MAX_ABS_TOL and rel <= REL_L2_TOL


def test_grouped_ffn_biases_few_rows():
    _say("ffn with biases, few rows")
    got, want = _ffn_case([5, 9], 1024, 4096, 4, 0, "f16", torch.float32, seed=6, with_bias=True)
    max_abs, rel = error_metrics(got, want)
    assert max_abs <= MAX_ABS_TOL and rel <= REL_L2_TOL


@pytest.mark.parametrize("rows,d,F,bits,g", [([5, 9], 1024, 4096, 4, 0),          # straight-line streaming kernels
                                              ([7, 0, 16], 512, 8192, 8, 0),       # run-loop streaming kernel (fc2)
                                              ([100, 260, 7], 256, 512, 4, 128)])  # tiled kernel, group scales
def test_grouped_ffn_gelu(rows, d, F, bits, g):
    _say(f"ffn with GELU rows={rows} d={d} F={F} bits={bits} g={g}")
    got, want = _ffn_case(rows, d, F, bits, g, "f16", torch.float32, seed=9, with_bias=True, activation="gelu")
    relu, _ = _ffn_case(rows, d, F, bits, g, "f16", torch.float32, seed=9, with_bias=True, activation="relu")
    max_abs, rel = error_metrics(got, want)
    _say(f"   max_abs={max_abs:.3e} rel_l2={rel:.3e}")
    assert max_abs <= MAX_ABS_TOL and rel <= REL_L2_TOL
    assert error_metrics(relu, want)[1] > 0.02                  # and it is not ReLU


def test_grouped_ffn_no_rows():
    _say("ffn R=0")
    off = torch.zeros(5, dtype=torch.int32, device=DEV)
    x = torch.empty((0, 128), dtype=torch.float16, device=DEV)
    w = torch.zeros((4, 128, 128), dtype=torch.float32, device=DEV)
    _, s, p = B.moe_quantize_experts(w, 4, 0, want_canon=False)
    y = B.moe_grouped_ffn_wq(x, off, 4, 128, 128, 4, 0, p, s, p, s)
    assert y.shape == (0, 128)


# ------------------------------------------------------------------ combine
@pytest.mark.parametrize("T,k,d,y_dt,o_dt", [(64, 2, 1024, torch.float16, torch.float32),
                                              (33, 1, 72, torch.float32, torch.float32),
                                              (50, 2, 128, torch.bfloat16, torch.float16),
                                              (7, 2, 64, torch.float32, torch.bfloat16)])
def test_combine_matches_oracle(T, k, d, y_dt, o_dt):
    _say(f"combine T={T} k={k} d={d} {y_dt}->{o_dt}")
    rng = np.random.default_rng(T + d)
    R = T * k
    y = to_dev(rng.standard_normal((R, d)).astype(np.float32), y_dt)
    inv = rng.permutation(R).astype(np.int32)
    scale = rng.uniform(0, 1, (T, k)).astype(np.float32)
    out = B.moe_combine(y, to_dev(inv, torch.int32), to_dev(scale, torch.float32), T, k, out_dtype=o_dt)
    torch.cuda.synchronize()
    want = oracle.round_to(oracle.combine(y.float().cpu().numpy(), inv, scale, T, k), oracle_dtype_code(o_dt))
    got = out.float().cpu().numpy()
    if o_dt == torch.float32:
        assert np.allclose(got, want, rtol=1e-6, atol=1e-6)
    else:
        ulp = 2.0 ** -10 if o_dt == torch.float16 else 2.0 ** -7
        assert np.all(np.abs(got - want) <= ulp * np.maximum(np.abs(want), 1e-3))


def test_calls_are_deterministic():
    _say("determinism")
    got1, _ = _ffn_case([12, 90, 31], 256, 512, 4, 0, "f16", torch.float16, seed=77)
    got2, _ = _ffn_case([12, 90, 31], 256, 512, 4, 0, "f16", torch.float16, seed=77)
    assert np.array_equal(got1, got2)


# ------------------------------------------------------------------ batch pruning (Sec. 3.5)
@pytest.mark.parametrize("T,d,E,k", [(64, 1024, 32, 2), (130, 192, 3, 1), (77, 2048, 128, 2), (16400, 128, 64, 2)])
def test_gate_marks_finished_rows(T, d, E, k):
    _say(f"gate with finished rows T={T} E={E} k={k}")
    rng = np.random.default_rng(T + E)
    x = to_dev(rng.standard_normal((T, d)).astype(np.float32), torch.float16)
    wg = to_dev((rng.standard_normal((d, E)) * 0.02).astype(np.float32), torch.float16)
    fin = (rng.random(T) < 0.35).astype(np.uint8)
    oi, osc = oracle.gate(x.float().cpu().numpy(), wg.float().cpu().numpy(), None, k, True, finished=fin)
    gi, gs = B.moe_gate_topk(x, wg, None, k, True, finished=to_dev(fin, torch.uint8))
    torch.cuda.synchronize()
    assert np.array_equal(gi.cpu().numpy(), oi)
    assert np.allclose(gs.cpu().numpy(), osc, rtol=1e-5, atol=1e-9)
    assert (oi[fin == 1] == E).all() and (oi[fin == 0] < E).all()


@pytest.mark.parametrize("T,k,E,d", [(64, 2, 32, 1024), (300, 2, 13, 128), (5000, 2, 128, 64), (16384, 1, 64, 256),
                                      (40, 1, 1, 64)])
def test_permute_with_pruned_rows_bit_exact(T, k, E, d):
    _say(f"permute with pruned rows T={T} k={k} E={E} d={d}")
    rng = np.random.default_rng(T + E + 1)
    idx = rng.integers(0, E, size=(T, k)).astype(np.int32)
    idx[rng.random(T) < 0.3] = E                                 # whole tokens pruned
    x = rng.standard_normal((T, d)).astype(np.float16)
    perm_src, inv_perm, off = oracle.permute(idx, E)
    xp, ps, ip, of = B.moe_permute(to_dev(idx, torch.int32), to_dev(x, torch.float16), E)
    torch.cuda.synchronize()
    assert np.array_equal(of.cpu().numpy(), off)
    assert np.array_equal(ps.cpu().numpy(), perm_src)
    assert np.array_equal(ip.cpu().numpy(), inv_perm)
    active = int(off[E])
    assert 0 < active < T * k
    assert np.array_equal(xp.cpu().numpy()[:active], x[perm_src[:active] // k])


def test_combine_skips_pruned_rows():
    _say("combine with pruned rows")
    rng = np.random.default_rng(12)
    T, k, d = 40, 2, 128
    R = T * k
    active = 51
    y = rng.standard_normal((R, d)).astype(np.float32)
    y[active:] = np.nan                                          # never computed: must not be read into the sum
    inv = rng.permutation(R).astype(np.int32)
    scale = rng.uniform(0, 1, (T, k)).astype(np.float32)
    act_dev = torch.tensor([active], dtype=torch.int32, device=DEV)
    out = B.moe_combine(to_dev(y, torch.float32), to_dev(inv, torch.int32), to_dev(scale, torch.float32), T, k,
                        active_rows=act_dev)
    torch.cuda.synchronize()
    want = oracle.combine(y, inv, scale, T, k, active_rows=active)
    got = out.cpu().numpy()
    assert np.isfinite(got).all() and np.allclose(got, want, rtol=1e-6, atol=1e-6)


# ------------------------------------------------------------------ single grouped GEMM (Table 1)
@pytest.mark.parametrize("bits,native,K,N", [(4, False, 1024, 256), (4, True, 1024, 256), (8, False, 1024, 192),
                                              (8, True, 1024, 192), (16, False, 1024, 256), (16, False, 512, 128),
                                              (16, False, 256, 64), (4, False, 4096, 128), (8, False, 512, 320)])
def test_grouped_gemm_matches_oracle(bits, native, K, N):
    _say(f"grouped gemm bits={bits} native={native} K={K} N={N}")
    rng = np.random.default_rng(bits + K + N + native)
    rows = [3, 0, 5, 1, 17, 2]
    E = len(rows)
    off = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    x = to_dev(rng.standard_normal((int(off[-1]), K)).astype(np.float32), torch.float16)
    w = (rng.standard_normal((E, K, N)) * 0.05).astype(np.float32)
    if bits == 16:
        packed = B.moe_pack_fp16_experts(to_dev(w, torch.float32))
        scales = None
        w_dq = w.astype(np.float16).astype(np.float32)
    else:
        _, scales, packed = B.moe_quantize_experts(to_dev(w, torch.float32), bits, 0, want_canon=False)
        q, s = oracle.quantize(w, bits, 0)
        w_dq = oracle.dequantize(q, s, 0)
    y = B.moe_grouped_gemm_wq(x, to_dev(off, torch.int32), E, K, N, bits, packed, scales, native_convert=native,
                              y_dtype=torch.float32)
    torch.cuda.synchronize()
    want = oracle.grouped_gemm(x.float().cpu().numpy(), off, w_dq)
    max_abs, rel = error_metrics(y.cpu().numpy(), want)
    _say(f"   max_abs={max_abs:.3e} rel_l2={rel:.3e}")
    assert max_abs <= MAX_ABS_TOL and rel <= 1e-5          # exact weights on both sides: only the fp32 summation order differs


# ------------------------------------------------------------------ routing fused into the GEMMs
@pytest.mark.parametrize("T,k,E,d,F,bits,g,o_dt", [
    (700, 1, 5, 128, 256, 4, 0, torch.float32), (300, 2, 3, 192, 320, 8, 0, torch.float32),
    (1500, 1, 4, 256, 512, 4, 128, torch.float32),
    # the fused un-permute storing 16-bit layer outputs
    (700, 1, 5, 128, 256, 4, 0, torch.float16), (650, 1, 3, 192, 320, 8, 0, torch.bfloat16),
    # rows fetched through the routing index by the 128-row tiles with a scale per group (K above 2048, 4-bit)
    (700, 1, 3, 2176, 2304, 4, 128, torch.float32), (400, 2, 3, 2112, 2176, 4, 64, torch.float32)])
def test_routed_ffn_matches_oracle(T, k, E, d, F, bits, g, o_dt):
    _say(f"routed ffn T={T} k={k} E={E} d={d} F={F} bits={bits} g={g} out={o_dt}")
    rng = np.random.default_rng(T + E + bits)
    x = rng.standard_normal((T, d)).astype(np.float16).astype(np.float32)
    wg = (rng.standard_normal((d, E)) * 0.05).astype(np.float16).astype(np.float32)
    w1 = (rng.standard_normal((E, d, F)) * 0.05).astype(np.float32)
    w2 = (rng.standard_normal((E, F, d)) * 0.05).astype(np.float32)
    q1, s1 = oracle.quantize(w1, bits, g)
    q2, s2 = oracle.quantize(w2, bits, g)
    res = oracle.moe_layer(x, wg, None, q1, s1, q2, s2, k, g, oracle.F16, y_dtype=oracle.F32)
    _, ds1, p1 = B.moe_quantize_experts(to_dev(w1, torch.float32), bits, g, want_canon=False)
    _, ds2, p2 = B.moe_quantize_experts(to_dev(w2, torch.float32), bits, g, want_canon=False)
    xd = to_dev(x, torch.float16)
    assert B.moe_grouped_ffn_wq_routed_supported(T * k, E, T, d, F, bits, g, torch.float16)
    idx, scale = B.moe_gate_topk(xd, to_dev(wg, torch.float16), None, k, True)
    assert np.array_equal(idx.cpu().numpy(), res["expert_idx"])
    # index only: no x_perm copy
    R = T * k
    ps = torch.empty(R, dtype=torch.int32, device=DEV)
    ip = torch.empty(R, dtype=torch.int32, device=DEV)
    of = torch.empty(E + 1, dtype=torch.int32, device=DEV)
    ws = torch.empty(B.moe_permute_workspace_bytes(T, k, E), dtype=torch.uint8, device=DEV)
    rc = B.load().moe_permute(idx.data_ptr(), None, 0, T, k, E, d, None, ps.data_ptr(), ip.data_ptr(), of.data_ptr(),
                              ws.data_ptr(), ws.numel(), None)
    assert rc == 0
    torch.cuda.synchronize()
    assert np.array_equal(ps.cpu().numpy(), res["perm_src"]) and np.array_equal(of.cpu().numpy(), res["expert_offsets"])
    if k == 1:      # gather and un-permute + scale fused: the call returns the layer output
        out = B.moe_grouped_ffn_wq_routed(xd, ps, k, of, E, d, F, bits, g, p1, ds1, p2, ds2, expert_scale=scale.view(-1),
                                          out_dtype=o_dt)
    else:           # gather fused; combine as usual
        y = B.moe_grouped_ffn_wq_routed(xd, ps, k, of, E, d, F, bits, g, p1, ds1, p2, ds2, out_dtype=torch.float32)
        out = B.moe_combine(y, ip, scale, T, k, out_dtype=o_dt)
    torch.cuda.synchronize()
    assert out.dtype == o_dt
    want = oracle.round_to(res["out"], oracle_dtype_code(o_dt))     # the layer output stored in o_dt: one rounding of the fp32 result
    max_abs, rel = error_metrics(out.float().cpu().numpy(), want)
    _say(f"   max_abs={max_abs:.3e} rel_l2={rel:.3e}")
    # a 16-bit output that lands on the other side of a rounding boundary differs by one unit in the last place
    ulp = {torch.float32: 0.0, torch.float16: 2.0 ** -10, torch.bfloat16: 2.0 ** -7}[o_dt] * float(np.abs(want).max())
    assert max_abs <= MAX_ABS_TOL + ulp and rel <= REL_L2_TOL + (1e-3 if o_dt == torch.bfloat16 else 0.0)


@pytest.mark.parametrize("T,k,E,d,F,bits,prune", [(64, 2, 32, 1024, 4096, 4, 0),     # the decode workload's shape
                                                   (40, 2, 5, 1024, 256, 4, 7),        # few experts: several row groups per expert, pruned rows
                                                   (256, 1, 8, 512, 2048, 8, 0),       # most assignments one launch takes
                                                   (37, 1, 9, 1024, 128, 8, 11),       # 8-bit slabs of 32 blocks, empty experts likely
                                                   (3, 2, 64, 2048, 128, 4, 1),        # 4-bit slabs of 32 blocks, nearly every expert empty
                                                   (64, 1, 1, 1024, 256, 4, 5),        # one expert takes every row: four row groups
                                                   (128, 2, 8, 512, 2048, 8, 0)])      # 256 assignments with two experts per token
def test_gated_ffn_matches_oracle(T, k, E, d, F, bits, prune):
    """Permutation rebuilt inside fc1: index arrays bit-exact with the oracle's stable sort, y_perm within tolerance."""
    _say(f"gated ffn T={T} k={k} E={E} d={d} F={F} bits={bits} pruned={prune}")
    rng = np.random.default_rng(T * 3 + E + bits + prune)
    x = rng.standard_normal((T, d)).astype(np.float16).astype(np.float32)
    wg = (rng.standard_normal((d, E)) * 0.05).astype(np.float16).astype(np.float32)
    w1 = (rng.standard_normal((E, d, F)) * 0.05).astype(np.float32)
    w2 = (rng.standard_normal((E, F, d)) * 0.05).astype(np.float32)
    finished = np.zeros(T, dtype=np.uint8)
    finished[rng.choice(T, size=prune, replace=False)] = 1
    q1, s1 = oracle.quantize(w1, bits, 0)
    q2, s2 = oracle.quantize(w2, bits, 0)
    idx_o, _ = oracle.gate(x, wg, None, k, True, finished=finished if prune else None)
    perm_src_o, inv_perm_o, off_o = oracle.permute(idx_o, E)
    active = int(off_o[E])
    x_perm_o = oracle.gather_rows(x, perm_src_o[:active], k)
    y_o = oracle.grouped_ffn(x_perm_o, off_o, q1, s1, q2, s2, 0, oracle.F16)
    _, ds1, p1 = B.moe_quantize_experts(to_dev(w1, torch.float32), bits, 0, want_canon=False)
    _, ds2, p2 = B.moe_quantize_experts(to_dev(w2, torch.float32), bits, 0, want_canon=False)
    xd = to_dev(x, torch.float16)
    level = B.moe_grouped_ffn_wq_gated_supported(T, k, E, d, F, bits, 0, torch.float16)
    assert level >= 1
    idx, scale = B.moe_gate_topk(xd, to_dev(wg, torch.float16), None, k, True, finished=to_dev(finished, torch.uint8) if prune else None)
    assert np.array_equal(idx.cpu().numpy(), idx_o)
    y, ps, ip, of = B.moe_grouped_ffn_wq_gated(xd, idx, E, d, F, bits, 0, p1, ds1, p2, ds2, y_dtype=torch.float32)
    torch.cuda.synchronize()
    assert np.array_equal(of.cpu().numpy(), off_o)
    assert np.array_equal(ps.cpu().numpy(), perm_src_o) and np.array_equal(ip.cpu().numpy(), inv_perm_o)
    max_abs, rel = error_metrics(y.cpu().numpy()[:active], y_o)
    _say(f"   active rows {active} of {T * k}; max_abs={max_abs:.3e} rel_l2={rel:.3e}")
    assert max_abs <= MAX_ABS_TOL and rel <= REL_L2_TOL
    if level == 2:      # un-permute fused in as well: fc2 adds the scaled rows into the layer output
        y_full = np.zeros((T * k, d), dtype=np.float32)
        y_full[:active] = y_o
        out_o = oracle.combine(y_full, inv_perm_o, scale.cpu().numpy(), T, k, active_rows=active)
        out1 = B.moe_grouped_ffn_wq_gated(xd, idx, E, d, F, bits, 0, p1, ds1, p2, ds2, expert_scale=scale)[0]
        out2 = B.moe_grouped_ffn_wq_gated(xd, idx, E, d, F, bits, 0, p1, ds1, p2, ds2, expert_scale=scale)[0]
        torch.cuda.synchronize()
        got = out1.cpu().numpy()
        assert np.array_equal(got, out2.cpu().numpy())               # the order of a token's two terms does not show
        assert not got[finished == 1].any()                          # pruned tokens: exactly zero
        max_abs, rel = error_metrics(got, out_o)
        _say(f"   un-permute fused: max_abs={max_abs:.3e} rel_l2={rel:.3e}")
        assert max_abs <= MAX_ABS_TOL and rel <= REL_L2_TOL


def _routing(kind, T, k, E, rng):
    """Expert indices [T, k] (distinct per token) for the decode-kernel cases."""
    idx = np.empty((T, k), dtype=np.int32)
    for t in range(T):
        if kind == "uniform":
            idx[t] = rng.choice(E, size=k, replace=False)
        elif kind == "one_hot_expert":          # expert 3 takes a row of every token: several passes of sixteen rows
            others = [e for e in range(E) if e != 3]
            idx[t] = ([3] + list(rng.choice(others, size=k - 1, replace=False)))[:k]
            if k == 2 and t % 2:
                idx[t] = idx[t][::-1]
        elif kind == "few_experts":             # most experts stay empty
            idx[t] = rng.choice(5, size=k, replace=False) * 3
    return idx


@pytest.mark.parametrize("T,k,E,d,F,bits,kind,extras", [
    (64, 2, 32, 1024, 4096, 4, "uniform", ""),                  # the decode workload's shape
    (64, 2, 32, 1024, 4096, 4, "one_hot_expert", ""),           # 64 rows in one expert: four passes; the rest one or two rows
    (30, 2, 32, 1024, 4096, 4, "few_experts", "pruned"),        # 27 experts without rows, pruned tokens
    (64, 2, 32, 1024, 4096, 4, "few_experts", "pruned"),        # the same with four assignments per expert: the weights are requested
                                                                # before the row counts are known, for 27 experts in vain
    (128, 2, 80, 1024, 2048, 4, "uniform", ""),                 # early requests and 320 items: some workgroups take two
    (64, 2, 32, 512, 2048, 8, "uniform", "bias gelu"),          # 8-bit weights, biases, GELU
    (1, 1, 64, 1024, 1024, 4, "uniform", ""),                   # a single row
    (128, 2, 136, 1024, 1024, 4, "uniform", ""),                # 272 items: some workgroups take two
    (50, 1, 16, 1024, 2048, 4, "one_hot_expert", "bias")])      # one expert per token, all fifty rows in one expert
def test_decode_ffn_matches_oracle(T, k, E, d, F, bits, kind, extras):
    """Decode-sized batches with the gate scale fused in: one streaming launch (sort, fc1, activation, fc2 per
    slice of d_ff) and the slice reduction.  Index arrays bit-exact, output within the layer tolerance, two
    calls bit-identical."""
    _say(f"decode ffn T={T} k={k} E={E} d={d} F={F} bits={bits} {kind} {extras}")
    rng = np.random.default_rng(T * 5 + E + bits + len(kind))
    x = rng.standard_normal((T, d)).astype(np.float16).astype(np.float32)
    w1 = (rng.standard_normal((E, d, F)) * 0.05).astype(np.float32)
    w2 = (rng.standard_normal((E, F, d)) * 0.05).astype(np.float32)
    idx = _routing(kind, T, k, E, rng)
    if "pruned" in extras:
        idx[rng.choice(T, size=7, replace=False)] = E
    scale = rng.uniform(0.1, 1.0, (T, k)).astype(np.float32)
    scale[idx == E] = 0.0
    ob1 = ob2 = b1 = b2 = None
    if "bias" in extras:
        ob1 = rng.standard_normal((E, F)).astype(np.float16).astype(np.float32) * 0.1
        ob2 = rng.standard_normal((E, d)).astype(np.float16).astype(np.float32) * 0.1
        b1, b2 = to_dev(ob1, torch.float16), to_dev(ob2, torch.float16)
    act = "gelu" if "gelu" in extras else "relu"
    q1, s1 = oracle.quantize(w1, bits, 0)
    q2, s2 = oracle.quantize(w2, bits, 0)
    perm_src_o, inv_perm_o, off_o = oracle.permute(idx, E)
    active = int(off_o[E])
    y_o = np.zeros((T * k, d), dtype=np.float32)
    y_o[:active] = oracle.grouped_ffn(oracle.gather_rows(x, perm_src_o[:active], k), off_o, q1, s1, q2, s2, 0, oracle.F16,
                                      ob1, ob2, activation=B.ACTIVATIONS[act])
    out_o = oracle.combine(y_o, inv_perm_o, scale, T, k, active_rows=active)
    _, ds1, p1 = B.moe_quantize_experts(to_dev(w1, torch.float32), bits, 0, want_canon=False)
    _, ds2, p2 = B.moe_quantize_experts(to_dev(w2, torch.float32), bits, 0, want_canon=False)
    assert B.moe_grouped_ffn_wq_gated_supported(T, k, E, d, F, bits, 0, torch.float16) == 2
    xd, idx_d, scale_d = to_dev(x, torch.float16), to_dev(idx, torch.int32), to_dev(scale, torch.float32)
    out1, ps, ip, of = B.moe_grouped_ffn_wq_gated(xd, idx_d, E, d, F, bits, 0, p1, ds1, p2, ds2, b1, b2, expert_scale=scale_d,
                                                  activation=act)
    assert B.load().moe_last_ffn_kernels().decode() == "decode_ffn_kernel"
    out2 = B.moe_grouped_ffn_wq_gated(xd, idx_d, E, d, F, bits, 0, p1, ds1, p2, ds2, b1, b2, expert_scale=scale_d, activation=act)[0]
    torch.cuda.synchronize()
    assert np.array_equal(of.cpu().numpy(), off_o)
    assert np.array_equal(ps.cpu().numpy(), perm_src_o) and np.array_equal(ip.cpu().numpy(), inv_perm_o)
    got = out1.cpu().numpy()
    assert np.array_equal(got, out2.cpu().numpy())
    assert not got[(idx == E).all(axis=1)].any()                # pruned tokens: exactly zero
    max_abs, rel = error_metrics(got, out_o)
    _say(f"   rows per expert up to {int(np.diff(off_o[:E + 1]).max())}, active {active} of {T * k}; max_abs={max_abs:.3e} rel_l2={rel:.3e}")
    assert max_abs <= MAX_ABS_TOL and rel <= REL_L2_TOL


def test_decode_kernel_alone_leaves_a_full_call_unchanged():
    """The gated call with a NULL output (the decode kernel without its slice reduction, which bench.py times) is
    accepted only where the decode kernel runs, and a full call after it gives the same bits as before it."""
    from paper_2211_10017_amd import MoEExpertLayer
    _say("decode kernel alone: NULL output accepted on the decode path only")
    T, k, E, d, F = 64, 2, 32, 1024, 1024
    rng = np.random.default_rng(77)
    layer = MoEExpertLayer(T, d, F, E, k, 4)
    for e in range(E):
        layer.load_expert(1, e, to_dev((rng.standard_normal((d, F)) * 0.05).astype(np.float32), torch.float32))
        layer.load_expert(2, e, to_dev((rng.standard_normal((F, d)) * 0.05).astype(np.float32), torch.float32))
    layer.wg.copy_(to_dev(rng.standard_normal((d, E)).astype(np.float32), torch.float16))
    x = to_dev(rng.standard_normal((T, d)).astype(np.float32), torch.float16)
    before = layer.forward(x).clone()
    assert B.load().moe_last_ffn_kernels().decode() == "decode_ffn_kernel"
    layer.out.fill_(7.0)
    layer.ffn_streaming_kernel_only(x)
    torch.cuda.synchronize()
    assert bool((layer.out == 7.0).all())                       # no reduction ran: the output buffer is untouched
    after = layer.forward(x)
    torch.cuda.synchronize()
    assert torch.equal(before, after)
    other = MoEExpertLayer(T, d, 1088, E, k, 4)                  # F not a multiple of 512: the streaming pair, not the decode kernel
    other.w1_packed.zero_(); other.w2_packed.zero_(); other.s1.zero_(); other.s2.zero_()
    other.wg.copy_(layer.wg)
    other.forward(x)
    with pytest.raises(B.MoeError):
        other.ffn_streaming_kernel_only(x)
    torch.cuda.synchronize()


def test_gated_ffn_refuses_other_sizes():
    _say("gated ffn: what the fused permutation does not take is refused")
    assert not B.moe_grouped_ffn_wq_gated_supported(512, 1, 8, 1024, 4096, 4, 0, torch.float16)      # more than 256 assignments
    assert not B.moe_grouped_ffn_wq_gated_supported(64, 2, 32, 1024, 4096, 4, 128, torch.float16)    # group scales
    assert not B.moe_grouped_ffn_wq_gated_supported(64, 2, 32, 1024, 4096, 4, 0, torch.bfloat16)     # bf16 rows
    assert not B.moe_grouped_ffn_wq_gated_supported(64, 2, 32, 4096, 4096, 4, 0, torch.float16)      # fc1 slabs of 64 blocks
    assert B.moe_grouped_ffn_wq_gated_supported(64, 2, 32, 1024, 4096, 4, 0, torch.float16) == 2
    assert B.moe_grouped_ffn_wq_gated_supported(64, 2, 32, 1024, 8192, 4, 0, torch.float16) == 1   # fc2's slabs too long for the fused un-permute


def test_routed_ffn_refuses_decode_sizes():
    _say("routed ffn: decode sizes are refused")
    assert not B.moe_grouped_ffn_wq_routed_supported(128, 32, 64, 1024, 4096, 4, 0, torch.float16)
    assert not B.moe_grouped_ffn_wq_routed_supported(16384, 64, 8192, 4096, 16384, 4, 128, torch.bfloat16)
    assert B.moe_grouped_ffn_wq_routed_supported(16384, 64, 8192, 4096, 16384, 4, 128, torch.float16)


# ------------------------------------------------------------------ limits and degenerate shapes
@pytest.mark.parametrize("T,d,E,k", [(3, 64, 256, 2), (5, 8, 2, 2), (1, 4096, 64, 1), (70, 72, 5, 1)])
def test_gate_limits(T, d, E, k):
    _say(f"gate limits T={T} d={d} E={E} k={k}")
    rng = np.random.default_rng(T * 7 + E)
    x = to_dev(rng.standard_normal((T, d)).astype(np.float32), torch.float16)
    wg = to_dev((rng.standard_normal((d, E)) * 0.1).astype(np.float32), torch.float16)
    oi, osc = oracle.gate(x.float().cpu().numpy(), wg.float().cpu().numpy(), None, k, True)
    gi, gs = B.moe_gate_topk(x, wg, None, k, True)
    torch.cuda.synchronize()
    assert np.array_equal(gi.cpu().numpy(), oi)
    assert np.allclose(gs.cpu().numpy(), osc, rtol=1e-5, atol=1e-9)


def test_permute_most_experts():
    _say("permute E=1024")
    rng = np.random.default_rng(77)
    T, k, E, d = 3000, 2, 1024, 64
    idx = rng.integers(0, E, size=(T, k)).astype(np.int32)
    x = rng.standard_normal((T, d)).astype(np.float16)
    perm_src, inv_perm, off = oracle.permute(idx, E)
    xp, ps, ip, of = B.moe_permute(to_dev(idx, torch.int32), to_dev(x, torch.float16), E)
    torch.cuda.synchronize()
    assert np.array_equal(of.cpu().numpy(), off) and np.array_equal(ps.cpu().numpy(), perm_src)
    assert np.array_equal(ip.cpu().numpy(), inv_perm) and np.array_equal(xp.cpu().numpy(), x[perm_src // k])


@pytest.mark.parametrize("rows,d,F,bits,g", [([1], 64, 64, 4, 0), ([1], 64, 64, 8, 64), ([0, 0, 2], 64, 128, 8, 0),
                                              ([128, 32, 64], 64, 64, 4, 0)])
def test_grouped_ffn_smallest_shapes(rows, d, F, bits, g):
    _say(f"ffn smallest shapes rows={rows} d={d} F={F} bits={bits} g={g}")
    got, want = _ffn_case(rows, d, F, bits, g, "f16", torch.float32, seed=3)
    max_abs, rel = error_metrics(got, want)
    assert max_abs <= MAX_ABS_TOL and rel <= REL_L2_TOL


def test_quantize_smallest_shape_and_extremes():
    _say("quantize K=64 N=32, huge and tiny weights")
    rng = np.random.default_rng(5)
    w = rng.standard_normal((2, 64, 32)).astype(np.float32)
    w[0, :, 0] *= 1e4                                            # scale near the top of fp16
    w[0, :, 1] *= 1e-7                                           # scale in the fp16 subnormals
    w[1, :, 2] = 0.0
    for bits in (4, 8):
        q, s, p = B.moe_quantize_experts(to_dev(w, torch.float32), bits, 0)
        torch.cuda.synchronize()
        oq, os_ = oracle.quantize(w, bits, 0)
        want_q = oq if bits == 8 else oracle.pack_int4(oq)
        assert np.array_equal(q.cpu().numpy(), want_q)
        assert np.array_equal(s.cpu().numpy().view(np.uint16), os_)
