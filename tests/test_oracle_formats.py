"""Pins for the oracle's number-format routines and the paper's I2F trick.

The fp16 / bf16 roundings are pinned to numpy's and torch's casts (library routines);
the magic-number conversion is pinned to the values the paper prints (tests/golden/) and to
plain integer conversion, exhaustively (Sec. 3.4.1 states the trick is exact).
"""
import os

import numpy as np
import torch

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_i2f_values.txt")


def _golden():
    out = {}
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, *vals = line.split()
        out[key] = [int(v, 0) for v in vals]
    return out


def test_f16_bits_roundtrip_all_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float32)
    for b in range(0, 65536, 7):          # stride keeps the ctypes loop short
        v = oracle.f16_bits_to_f32(int(b))
        if np.isnan(ref[b]):
            assert np.isnan(v)
        else:
            assert v == ref[b], hex(b)
            assert oracle.f32_to_f16_bits(float(ref[b])) == b or ref[b] == 0.0


def test_round_f16_matches_numpy_cast():
    rng = np.random.default_rng(0)
    vals = np.concatenate([
        rng.standard_normal(200000).astype(np.float32),
        (rng.standard_normal(50000) * 1e-6).astype(np.float32),       # subnormal range
        (rng.standard_normal(50000) * 3e4).astype(np.float32),        # near overflow
        np.array([0.0, -0.0, 65504.0, 65519.9, 65520.0, 70000.0, -65520.0, 2.0 ** -24, 2.0 ** -25,
                  1.5 * 2.0 ** -24, 2.5 * 2.0 ** -24, 2.0 ** -14, 2.0 ** -14 - 2.0 ** -25,
                  1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 2047.5, 2048.5, np.inf, -np.inf],
                 dtype=np.float32)])
    with np.errstate(over="ignore"):
        ref = vals.astype(np.float16).astype(np.float32)
    got = oracle.round_to(vals, oracle.F16)
    assert np.array_equal(got, ref)
    assert np.array_equal(np.signbit(got), np.signbit(ref))


def test_round_bf16_matches_torch_cast():
    rng = np.random.default_rng(1)
    vals = np.concatenate([
        rng.standard_normal(200000).astype(np.float32),
        (rng.standard_normal(50000) * 1e-30).astype(np.float32),
        (rng.standard_normal(50000) * 1e30).astype(np.float32),
        np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -9, 3.3895313e38, np.inf, 0.0],
                 dtype=np.float32)])
    ref = torch.from_numpy(vals).to(torch.bfloat16).to(torch.float32).numpy()
    got = oracle.round_to(vals, oracle.BF16)
    assert np.array_equal(got, ref)


def test_paper_printed_fp16_patterns():
    g = _golden()
    assert oracle.f32_to_f16_bits(1027.0) == g["fp16_bits_of_1027"][0]
    assert oracle.f32_to_f16_bits(1024.0) == g["fp16_bits_of_1024"][0]
    assert oracle.f16_bits_to_f32(g["fp16_bits_of_1027"][0]) == 1027.0
    # observation 1: for 1024 <= X < 2048 the mantissa field holds int(X - 1024)
    for x in range(1024, 2048):
        assert oracle.f32_to_f16_bits(float(x)) & 0x3ff == x - 1024
        assert oracle.f32_to_f16_bits(float(x)) >> 10 == g["fp16_bits_of_1024"][0] >> 10


def test_i2f_magic_is_exact_for_every_code():
    g = _golden()
    for bits, off_key, sub_key in ((8, "int8_offset", "int8_subtrahend"), (4, "int4_offset", "int4_subtrahend")):
        offset = g[off_key][0]
        assert g[sub_key][0] == 1024 + offset
        for code_plus in range(1 << bits):
            biased, res = oracle.i2f_magic(code_plus, offset)
            # observation 2: OR into 0x6400 builds the FP16 number 1024 + Y
            assert biased == (g["fp16_bits_of_1024"][0] | code_plus)
            assert np.uint16(biased).view(np.float16) == np.float16(1024 + code_plus)
            # exact against plain integer-to-float conversion of the signed code
            signed = code_plus - offset
            assert np.uint16(res).view(np.float16) == np.float16(signed)
            assert float(np.uint16(res).view(np.float16)) == float(signed)
    # outside the stated domain (Y >= 1024) the OR no longer adds: the trick must not be used
    assert g["magic_domain"][0] == 1024


def test_int4_interleave_order():
    g = _golden()
    src = np.array([10, 11, 12, 13, 14, 15, 16, 17], dtype=np.int8)
    out = oracle.int4_interleave8(src)
    assert list(out) == [int(src[i]) for i in g["int4_interleave"]]
