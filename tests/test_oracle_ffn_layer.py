"""Pins for the oracle's expert FFN, combine and whole layer (Sec. 3.3-3.4): the E=1 case
against a dense FFN through a library matmul, a tiny brute force in Python floats, the
dense-masked formulation, and invariants of the routing."""
import itertools

import numpy as np
import pytest

import oracle


def _layer_inputs(T, d, F, E, bits, g, seed, act=np.float16):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, d)).astype(act).astype(np.float32)
    wg = (rng.standard_normal((d, E)) * 0.05).astype(act).astype(np.float32)
    w1 = (rng.standard_normal((E, d, F)) * 0.05).astype(np.float32)
    w2 = (rng.standard_normal((E, F, d)) * 0.05).astype(np.float32)
    q1, s1 = oracle.quantize(w1, bits, g)
    q2, s2 = oracle.quantize(w2, bits, g)
    return x, wg, q1, s1, q2, s2


@pytest.mark.parametrize("bits,g", [(8, 0), (4, 0), (4, 16)])
def test_single_expert_equals_dense_ffn_via_library_matmul(bits, g):
    T, d, F = 24, 64, 48                      # d != F: a transposed operand cannot pass
    x, wg, q1, s1, q2, s2 = _layer_inputs(T, d, F, 1, bits, g, seed=bits + g)
    res = oracle.moe_layer(x, wg, None, q1, s1, q2, s2, k=1, group_size=g, act_dtype=oracle.F16)
    assert np.array_equal(res["expert_scale"], np.ones((T, 1), dtype=np.float32))
    assert np.array_equal(res["perm_src"], np.arange(T))
    w1 = oracle.dequantize(q1, s1, g)[0].astype(np.float64)
    w2 = oracle.dequantize(q2, s2, g)[0].astype(np.float64)
    h = np.maximum(x.astype(np.float64) @ w1, 0.0).astype(np.float16).astype(np.float64)
    y = h @ w2
    assert np.allclose(res["out"], y, rtol=1e-6, atol=1e-6)
    assert np.abs(y).max() > 0.1


def test_ffn_biases_relu_and_h_rounding():
    rng = np.random.default_rng(5)
    m, d, F = 6, 32, 40
    x = rng.standard_normal((m, d)).astype(np.float32)
    w1 = rng.standard_normal((d, F)).astype(np.float32)
    w2 = rng.standard_normal((F, d)).astype(np.float32)
    b1 = rng.standard_normal(F).astype(np.float32)
    b2 = rng.standard_normal(d).astype(np.float32)
    for act, npcast in ((oracle.F16, lambda a: a.astype(np.float16).astype(np.float64)),
                        (oracle.F32, lambda a: a.astype(np.float32).astype(np.float64))):
        y, h = oracle.expert_ffn(x, w1, w2, act, b1, b2, return_h=True)
        href = npcast(np.maximum(x.astype(np.float64) @ w1.astype(np.float64) + b1, 0.0))
        assert np.array_equal(h.astype(np.float64), href)
        assert (h == 0).sum() > m * F // 4 and (h > 0).sum() > m * F // 4
        assert np.allclose(y, href @ w2.astype(np.float64) + b2, rtol=1e-6, atol=1e-5)
    import torch
    y, h = oracle.expert_ffn(x, w1, w2, oracle.BF16, return_h=True)
    href = np.maximum(x.astype(np.float64) @ w1.astype(np.float64), 0.0).astype(np.float32)
    assert np.array_equal(h, torch.from_numpy(href).to(torch.bfloat16).float().numpy())


def test_tiny_layer_brute_force_in_python_floats():
    # T=4 tokens, E=3 experts, k=2, d=64 (one gate block), F=8: every number recomputed with
    # Python floats (fp64) straight from the definitions
    T, d, F, E, k = 4, 64, 8, 3, 2
    x, wg, q1, s1, q2, s2 = _layer_inputs(T, d, F, E, 8, 0, seed=11)
    res = oracle.moe_layer(x, wg, None, q1, s1, q2, s2, k=k, group_size=0, act_dtype=oracle.F16)
    sf1, sf2 = oracle.scales_to_f32(s1), oracle.scales_to_f32(s2)
    for t in range(T):
        logit = [sum(float(x[t, i]) * float(wg[i, e]) for i in range(d)) for e in range(E)]
        top = sorted(range(E), key=lambda e: (-logit[e], e))[:k]
        assert list(res["expert_idx"][t]) == top
        pe = [np.exp(l - max(logit)) for l in logit]
        sel = [pe[e] / sum(pe) for e in top]
        gate = [v / sum(sel) for v in sel]
        out = [0.0] * d
        for j, e in enumerate(top):
            h = []
            for n in range(F):
                acc = sum(float(x[t, i]) * (float(q1[e, i, n]) * float(sf1[e, 0, n])) for i in range(d))
                h.append(float(np.float16(max(acc, 0.0))))
            for n in range(d):
                yv = sum(h[i] * (float(q2[e, i, n]) * float(sf2[e, 0, n])) for i in range(F))
                out[n] += gate[j] * yv
        assert np.allclose(res["expert_scale"][t], gate, rtol=1e-6)
        assert np.allclose(res["out"][t], out, rtol=1e-5, atol=1e-6)


@pytest.mark.parametrize("k", [1, 2])
def test_dense_masked_formulation_matches_sorted_formulation(k):
    T, d, F, E = 96, 128, 64, 5
    x, wg, q1, s1, q2, s2 = _layer_inputs(T, d, F, E, 4, 0, seed=20 + k)
    a = oracle.moe_layer(x, wg, None, q1, s1, q2, s2, k=k, group_size=0, act_dtype=oracle.F16)
    b = oracle.moe_layer_dense_masked(x, wg, None, q1, s1, q2, s2, k=k, group_size=0, act_dtype=oracle.F16)
    assert np.allclose(a["out"], b, rtol=1e-6, atol=1e-7)
    # routing invariants
    counts = np.diff(a["expert_offsets"])
    assert counts.sum() == T * k and a["expert_offsets"][0] == 0
    assert np.array_equal(np.bincount(a["perm_src"] // k, minlength=T), np.full(T, k))
    assert np.array_equal(a["x_perm"], x[a["perm_src"] // k])
    if k == 2:
        assert np.all(a["expert_idx"][:, 0] != a["expert_idx"][:, 1])


def test_output_is_invariant_to_row_order_within_an_expert():
    T, d, F, E, k = 40, 64, 32, 3, 1
    x, wg, q1, s1, q2, s2 = _layer_inputs(T, d, F, E, 8, 0, seed=31)
    a = oracle.moe_layer(x, wg, None, q1, s1, q2, s2, k=k, group_size=0, act_dtype=oracle.F16)
    rng = np.random.default_rng(0)
    perm_src, off = a["perm_src"].copy(), a["expert_offsets"]
    for e in range(E):
        seg = perm_src[off[e]:off[e + 1]]
        perm_src[off[e]:off[e + 1]] = rng.permutation(seg)
    inv = np.empty_like(perm_src)
    inv[perm_src] = np.arange(perm_src.size, dtype=np.int32)
    xp = oracle.gather_rows(x, perm_src, k)
    y = oracle.grouped_ffn(xp, off, q1, s1, q2, s2, 0, oracle.F16)
    out = oracle.combine(y, inv, a["expert_scale"], T, k)
    assert np.array_equal(out, a["out"])


def test_grouped_ffn_row_subset_is_exact():
    T, d, F, E, k = 64, 64, 32, 4, 2
    x, wg, q1, s1, q2, s2 = _layer_inputs(T, d, F, E, 4, 16, seed=41)
    a = oracle.moe_layer(x, wg, None, q1, s1, q2, s2, k=k, group_size=16, act_dtype=oracle.F16)
    rows = np.array([0, 3, 17, 64, 100, 127])
    y = oracle.grouped_ffn(a["x_perm"], a["expert_offsets"], q1, s1, q2, s2, 16, oracle.F16, rows=rows)
    assert np.array_equal(y[rows], a["y_perm"][rows])
    rest = np.setdiff1d(np.arange(T * k), rows)
    assert not y[rest].any()


def test_combine_closed_form():
    # y rows are constant vectors equal to their row number; scale picks known weights
    T, k, d = 3, 2, 4
    y = np.repeat(np.arange(6, dtype=np.float32)[:, None], d, axis=1)
    inv = np.array([5, 0, 1, 4, 2, 3], dtype=np.int32)
    scale = np.array([[0.25, 0.75], [1.0, 0.0], [0.5, 0.5]], dtype=np.float32)
    out = oracle.combine(y, inv, scale, T, k)
    assert np.array_equal(out[:, 0], np.array([0.25 * 5 + 0, 1.0, 2.5], dtype=np.float32))


def test_grouped_gemm_against_library_matmul():
    """The single grouped GEMM (Table 1's operation) against a library fp64 matmul per expert;
    K != N and uneven row counts, so a transposed operand or a shifted offset cannot pass."""
    rng = np.random.default_rng(21)
    rows = [3, 0, 5, 1]
    K, N = 24, 40
    off = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    x = rng.standard_normal((off[-1], K)).astype(np.float16).astype(np.float32)
    w = rng.standard_normal((len(rows), K, N)).astype(np.float32)
    got = oracle.grouped_gemm(x, off, w)
    for e in range(len(rows)):
        want = x[off[e]:off[e + 1]].astype(np.float64) @ w[e].astype(np.float64)
        assert np.allclose(got[off[e]:off[e + 1]], want, rtol=1e-6, atol=1e-6)
    assert np.abs(got).max() > 1.0


def test_gelu_against_library_gelu():
    """The second activation (exact GELU) against torch's CPU implementation in fp64, through a
    one-expert FFN whose second matrix is the identity, so that y is h itself."""
    import torch
    rng = np.random.default_rng(31)
    m, d = 16, 32
    x = (rng.standard_normal((m, d)) * 2.0).astype(np.float32)
    eye = np.eye(d, dtype=np.float32)
    y, h = oracle.expert_ffn(x, eye, eye, oracle.F32, return_h=True, activation=oracle.GELU)
    want = torch.nn.functional.gelu(torch.from_numpy(x).double()).numpy()
    assert np.allclose(h, want, rtol=1e-6, atol=1e-7) and np.allclose(y, want, rtol=1e-6, atol=1e-7)
    assert (h[x < -1.0] < 0).all() and not np.allclose(h, np.maximum(x, 0.0), atol=1e-3)   # it is not ReLU
    relu = oracle.expert_ffn(x, eye, eye, oracle.F32, activation=oracle.RELU)
    assert np.array_equal(relu, np.maximum(x, 0.0))
