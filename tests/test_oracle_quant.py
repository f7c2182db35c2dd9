"""Pins for the oracle's quantiser and Algorithm 1 (Sec. 3.4): hand-worked columns,
invariants of symmetric range-based quantisation, and exactness of q*s."""
import numpy as np
import pytest

import oracle


def test_hand_worked_int4_column():
    # one expert, K=8, N=2.  Column 0: amax = 7/32 so the scale is exactly 2^-5 and the codes
    # can be read off; 2.5 and 3.5 steps are ties and go to the even code.
    s = 2.0 ** -5
    col0 = np.array([7, -7, 2.5, 3.5, -2.5, 0.49, -0.51, 0], dtype=np.float64) * s
    col1 = np.zeros(8)                                   # all-zero channel
    w = np.stack([col0, col1], axis=1)[None].astype(np.float32)
    q, sb = oracle.quantize(w, 4)
    assert sb.shape == (1, 1, 2)
    assert oracle.scales_to_f32(sb)[0, 0, 0] == np.float32(s)
    assert list(q[0, :, 0]) == [7, -7, 2, 4, -2, 0, -1, 0]
    assert oracle.scales_to_f32(sb)[0, 0, 1] == 0.0 and not q[0, :, 1].any()
    assert np.array_equal(oracle.dequantize(q, sb)[0, :, 0],
                          np.array([7, -7, 2, 4, -2, 0, -1, 0], dtype=np.float32) * np.float32(s))


def test_hand_worked_int8_column_uses_fp16_rounded_scale():
    # amax = 0.7: 0.7/127 is not an fp16 number; the stored scale is its fp16 rounding and the
    # codes divide by that stored value (so the largest element may land on 127 or 126.99..)
    w = np.array([0.7, -0.35, 0.1, 0.0055], dtype=np.float32).reshape(1, 4, 1)
    q, sb = oracle.quantize(w, 8)
    s = float.fromhex("0x1.694p-8")                      # fp16 nearest to 0.7/127 = 0.0055118...: 0.00551223754...
    assert float(oracle.scales_to_f32(sb)[0, 0, 0]) == s
    assert float(np.float16(np.float32(0.7) / np.float32(127))) == s
    # w/s = 126.990, -63.495, 18.141, 0.9978  (0.35/0.0055118 would have been 63.5: the
    # division is by the stored scale, not by amax/127)
    assert list(q.ravel()) == [127, -63, 18, 1]


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("g", [0, 16])
def test_quantizer_invariants(bits, g):
    rng = np.random.default_rng(bits * 10 + g)
    E, K, N = 3, 64, 24
    w = (rng.standard_normal((E, K, N)) * 0.02).astype(np.float32)
    w[1, :, 5] = 0.0                                       # a dead channel
    q, sb = oracle.quantize(w, bits, g)
    gg = K if g == 0 else g
    qmax = 2 ** (bits - 1) - 1
    s = oracle.scales_to_f32(sb)
    assert q.dtype == np.int8 and np.abs(q).max() <= qmax
    # every non-zero (channel, group) uses the full range
    qa = np.abs(q.reshape(E, K // gg, gg, N)).max(axis=2)
    assert np.array_equal(qa[s > 0], np.full((s > 0).sum(), qmax))
    assert not qa[s == 0].any()
    # the scale is the fp16 rounding of amax/qmax
    amax = np.abs(w.reshape(E, K // gg, gg, N)).max(axis=2)
    assert np.array_equal(s, (amax / np.float32(qmax)).astype(np.float16).astype(np.float32))
    # round-to-nearest: reconstruction error at most half a step (plus the clamp at the top code)
    wdq = oracle.dequantize(q, sb, g)
    step = np.repeat(s, gg, axis=1)
    assert np.all(np.abs(w - wdq) <= 0.5 * step * (1 + 1e-6) + np.abs(w) * 1e-3)
    # idempotent: quantising the dequantised weights gives the same codes and scales
    q2, sb2 = oracle.quantize(wdq, bits, g)
    assert np.array_equal(q2, q) and np.array_equal(sb2, sb)
    # sign symmetry
    q3, sb3 = oracle.quantize(-w, bits, g)
    assert np.array_equal(q3, -q) and np.array_equal(sb3, sb)


def test_group_size_K_equals_per_channel():
    rng = np.random.default_rng(7)
    w = rng.standard_normal((2, 32, 8)).astype(np.float32)
    qa, sa = oracle.quantize(w, 4, 0)
    qb, sb = oracle.quantize(w, 4, 32)
    assert np.array_equal(qa, qb) and np.array_equal(sa, sb) and sa.shape == (2, 1, 8)


def test_channel_axis_is_N_and_groups_run_along_K():
    # scales (E,1,N) for weights (E,M,N): scaling one output column must change only its scale
    rng = np.random.default_rng(8)
    w = rng.standard_normal((1, 16, 4)).astype(np.float32)
    _, s0 = oracle.quantize(w, 8)
    w2 = w.copy()
    w2[0, :, 2] *= 4.0
    q2, s2 = oracle.quantize(w2, 8)
    f0, f2 = oracle.scales_to_f32(s0), oracle.scales_to_f32(s2)
    assert np.array_equal(f2[0, 0, [0, 1, 3]], f0[0, 0, [0, 1, 3]]) and f2[0, 0, 2] == 4 * f0[0, 0, 2]
    # with groups of 8 rows, scaling rows 8..15 changes only group 1
    w3 = w.copy()
    w3[0, 8:, :] *= 2.0
    _, s3 = oracle.quantize(w3, 8, 8)
    _, s1 = oracle.quantize(w, 8, 8)
    assert np.array_equal(s3[0, 0], s1[0, 0]) and not np.array_equal(s3[0, 1], s1[0, 1])


def test_dequantize_is_exact_product():
    # Algorithm 1: f * S[e, n]; an 8-bit integer times an 11-bit significand fits in 24 bits
    rng = np.random.default_rng(9)
    q = rng.integers(-127, 128, size=(2, 32, 16)).astype(np.int8)
    sb = rng.integers(0x0001, 0x7bff, size=(2, 2, 16)).astype(np.uint16)     # any finite positive fp16
    wdq = oracle.dequantize(q, sb, 16)
    s64 = sb.view(np.float16).astype(np.float64)
    exact = q.astype(np.float64) * np.repeat(s64, 16, axis=1)
    assert np.array_equal(wdq.astype(np.float64), exact)


def test_int4_pack_roundtrip_and_nibble_order():
    q = np.array([[-7, 7, 0, -1, 3, -8 + 1, 5, 2]], dtype=np.int8)
    b = oracle.pack_int4(q)
    assert b.shape == (1, 4)
    assert b[0, 0] == ((7 << 4) | (-7 & 0xf)) and b[0, 1] == ((0xf << 4) | 0)   # even n low nibble
    assert np.array_equal(oracle.unpack_int4(b), q)
