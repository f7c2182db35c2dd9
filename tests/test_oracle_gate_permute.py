"""Pins for the oracle's gate and routing (Sec. 3.3): closed forms, library softmax/argsort,
fp64 logits, and the permutation invariants."""
import numpy as np
import scipy.special

import oracle


def _rand_inputs(T, d, E, seed):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, d)).astype(np.float16).astype(np.float32)
    wg = (rng.standard_normal((d, E)) * 0.02).astype(np.float16).astype(np.float32)
    return x, wg


def test_equal_logits_pick_lowest_experts_with_uniform_scale():
    x = np.ones((5, 64), dtype=np.float32)
    wg = np.zeros((64, 6), dtype=np.float32)
    idx, sc = oracle.gate(x, wg, None, 1)
    assert np.array_equal(idx, np.zeros((5, 1))) and np.allclose(sc, 1 / 6, rtol=1e-7)
    idx, sc = oracle.gate(x, wg, None, 2, renormalize=True)
    assert np.array_equal(idx, np.tile([0, 1], (5, 1))) and np.allclose(sc, 0.5, rtol=1e-7)
    idx, sc = oracle.gate(x, wg, None, 2, renormalize=False)
    assert np.allclose(sc, 1 / 6, rtol=1e-7)


def test_one_hot_gate_weight_gives_known_argmax_and_softmax():
    # token t has a single non-zero feature t; Wg row t has value 1 at expert (3t+1) % E
    T, d, E = 8, 64, 5
    x = np.zeros((T, d), dtype=np.float32)
    wg = np.zeros((d, E), dtype=np.float32)
    for t in range(T):
        x[t, t] = 2.0
        wg[t, (3 * t + 1) % E] = 1.0
    idx, sc, lg = oracle.gate(x, wg, None, 1, return_logits=True)
    assert list(idx[:, 0]) == [(3 * t + 1) % E for t in range(T)]
    assert np.allclose(sc[:, 0], np.exp(2.0) / (np.exp(2.0) + (E - 1)), rtol=1e-6)
    assert np.array_equal(lg.sum(axis=1), np.full(T, 2.0, dtype=np.float32))
    # a bias large enough moves every token to expert 4
    bias = np.array([0, 0, 0, 0, 5], dtype=np.float32)
    idx, _ = oracle.gate(x, wg, bias, 1)
    assert np.all(idx == 4)


def test_single_expert():
    x, wg = _rand_inputs(7, 128, 1, 0)
    idx, sc = oracle.gate(x, wg, None, 1)
    assert not idx.any() and np.array_equal(sc, np.ones((7, 1), dtype=np.float32))


def test_logits_and_scales_against_fp64_and_library_softmax():
    T, d, E, k = 64, 640, 24, 2           # d = 5 blocks of 128: exercises the partial-sum order
    x, wg = _rand_inputs(T, d, E, 1)
    bias = np.linspace(-0.3, 0.3, E).astype(np.float32)
    idx, sc, lg = oracle.gate(x, wg, bias, k, renormalize=True, return_logits=True)
    ref = x.astype(np.float64) @ wg.astype(np.float64) + bias
    assert np.allclose(lg, ref, rtol=0, atol=2e-5)
    order = np.argsort(-ref, axis=1, kind="stable")[:, :k]
    gap = np.sort(ref, axis=1)[:, -k] - np.sort(ref, axis=1)[:, -k - 1]
    clear = gap > 1e-4                      # where fp32 rounding cannot flip the choice
    assert clear.sum() > T // 2
    assert np.array_equal(idx[clear], order[clear])
    p = scipy.special.softmax(lg.astype(np.float64), axis=1)
    psel = np.take_along_axis(p, idx.astype(np.int64), axis=1)
    assert np.allclose(sc, psel / psel.sum(axis=1, keepdims=True), rtol=1e-6)
    assert np.allclose(sc.sum(axis=1), 1.0, rtol=1e-6)
    assert np.all(sc[:, 0] >= sc[:, 1])     # slots in descending logit order
    idx1, sc1 = oracle.gate(x, wg, bias, 1)
    assert np.array_equal(idx1[:, 0], idx[:, 0])
    assert np.allclose(sc1[:, 0], np.take_along_axis(p, idx1.astype(np.int64), axis=1)[:, 0], rtol=1e-6)
    _, scn = oracle.gate(x, wg, bias, 2, renormalize=False)
    assert np.allclose(scn, psel, rtol=1e-6)


def test_logit_summation_order_is_the_stated_one():
    # values chosen so that float addition order matters: the result must equal the stated
    # four-partial-sum order evaluated with numpy float32 scalars
    rng = np.random.default_rng(3)
    d = 1024
    x = (rng.standard_normal((1, d)) * np.exp(rng.uniform(-6, 6, d))).astype(np.float16).astype(np.float32)
    wg = rng.standard_normal((d, 3)).astype(np.float16).astype(np.float32)
    _, _, lg = oracle.gate(x, wg, None, 1, return_logits=True)
    for e in range(3):
        p = [np.float32(0)] * 4
        for i in range(d):
            p[(i // 128) % 4] = np.float32(p[(i // 128) % 4] + np.float32(x[0, i] * wg[i, e]))
        want = np.float32(np.float32(np.float32(p[0] + p[1]) + p[2]) + p[3])
        assert lg[0, e] == want


def test_ties_go_to_lower_expert_index():
    x = np.ones((1, 64), dtype=np.float32)
    wg = np.zeros((64, 4), dtype=np.float32)
    wg[0, 1] = wg[0, 3] = 1.0
    idx, sc = oracle.gate(x, wg, None, 2)
    assert list(idx[0]) == [1, 3] and np.allclose(sc, 0.5)


def test_permute_matches_stable_argsort_and_invariants():
    rng = np.random.default_rng(4)
    T, k, E = 300, 2, 13
    idx = rng.integers(0, E - 2, size=(T, k)).astype(np.int32)      # experts 11, 12 stay empty
    perm_src, inv_perm, off = oracle.permute(idx, E)
    flat = idx.ravel()
    assert np.array_equal(perm_src, np.argsort(flat, kind="stable"))
    assert np.array_equal(off, np.concatenate([[0], np.cumsum(np.bincount(flat, minlength=E))]))
    assert off[-1] == T * k and off[E - 1] == off[E] == off[E - 2]
    assert np.array_equal(np.sort(perm_src), np.arange(T * k))
    assert np.array_equal(inv_perm[perm_src], np.arange(T * k))
    assert np.array_equal(perm_src[inv_perm], np.arange(T * k))
    sorted_e = flat[perm_src]
    assert np.all(np.diff(sorted_e) >= 0)
    same = np.diff(sorted_e) == 0
    assert np.all(np.diff(perm_src)[same] > 0)                       # stable within an expert
    assert np.array_equal(np.bincount(perm_src // k, minlength=T), np.full(T, k))
    x = rng.standard_normal((T, 8)).astype(np.float32)
    assert np.array_equal(oracle.gather_rows(x, perm_src, k), x[perm_src // k])


def test_permute_empty_and_single():
    perm_src, inv_perm, off = oracle.permute(np.zeros((0, 1), dtype=np.int32), 4)
    assert perm_src.size == 0 and list(off) == [0, 0, 0, 0, 0]
    perm_src, inv_perm, off = oracle.permute(np.array([[2]], dtype=np.int32), 4)
    assert list(perm_src) == [0] and list(off) == [0, 0, 0, 1, 1]
