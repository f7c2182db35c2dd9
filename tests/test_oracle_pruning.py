"""Pins for the oracle's batch pruning (Sec. 3.5): rows of finished sentences get an expert index
past the real experts, sort behind every active row and are not processed.  The pins do not come
from the pruning code itself: a pruned layer must equal the un-pruned layer run on the
surviving tokens alone, and the index arrays must equal a library stable sort."""
import numpy as np
import pytest

import oracle
from test_oracle_ffn_layer import _layer_inputs


@pytest.mark.parametrize("k,bits,g", [(1, 8, 0), (2, 4, 0), (2, 4, 32)])
def test_pruned_layer_equals_layer_on_surviving_tokens(k, bits, g):
    T, d, F, E = 37, 64, 96, 5
    x, wg, q1, s1, q2, s2 = _layer_inputs(T, d, F, E, bits, g, seed=11 * k + bits)
    rng = np.random.default_rng(3)
    finished = (rng.random(T) < 0.4).astype(np.uint8)
    finished[0], finished[1] = 1, 0              # both kinds present
    res = oracle.moe_layer(x, wg, None, q1, s1, q2, s2, k=k, group_size=g, act_dtype=oracle.F16, finished=finished)
    keep = np.flatnonzero(finished == 0)
    ref = oracle.moe_layer(x[keep], wg, None, q1, s1, q2, s2, k=k, group_size=g, act_dtype=oracle.F16)
    assert np.array_equal(res["out"][keep], ref["out"])          # rows are independent: bit-identical
    assert not res["out"][finished == 1].any()                   # pruned rows are exactly zero
    assert np.abs(ref["out"]).max() > 0.05
    # routing of the survivors is untouched, pruned rows carry index E and scale 0
    assert np.array_equal(res["expert_idx"][keep], ref["expert_idx"])
    assert np.array_equal(res["expert_scale"][keep], ref["expert_scale"])
    assert (res["expert_idx"][finished == 1] == E).all() and not res["expert_scale"][finished == 1].any()
    # the number of active rows and the per-expert counts are those of the surviving tokens
    assert res["expert_offsets"][E] == keep.size * k
    assert np.array_equal(np.diff(res["expert_offsets"]), np.diff(ref["expert_offsets"]))


def test_permute_with_pruned_rows_matches_library_stable_sort():
    rng = np.random.default_rng(8)
    T, k, E = 50, 2, 7
    idx = rng.integers(0, E, size=(T, k)).astype(np.int32)
    idx[rng.random(T) < 0.3] = E                                   # whole tokens pruned
    perm_src, inv_perm, offsets = oracle.permute(idx, E)
    flat = idx.reshape(-1)
    assert np.array_equal(perm_src, np.argsort(flat, kind="stable"))
    assert np.array_equal(inv_perm[perm_src], np.arange(T * k))
    assert np.array_equal(offsets, np.concatenate([[0], np.cumsum(np.bincount(flat, minlength=E + 1)[:E])]))
    assert offsets[E] == (flat < E).sum()
    assert (flat[perm_src[offsets[E]:]] == E).all()


def test_all_rows_pruned_and_none_pruned():
    T, d, F, E = 9, 64, 64, 3
    x, wg, q1, s1, q2, s2 = _layer_inputs(T, d, F, E, 8, 0, seed=2)
    none = oracle.moe_layer(x, wg, None, q1, s1, q2, s2, k=1, group_size=0, act_dtype=oracle.F16,
                            finished=np.zeros(T, dtype=np.uint8))
    plain = oracle.moe_layer(x, wg, None, q1, s1, q2, s2, k=1, group_size=0, act_dtype=oracle.F16)
    assert np.array_equal(none["out"], plain["out"]) and np.array_equal(none["perm_src"], plain["perm_src"])
    every = oracle.moe_layer(x, wg, None, q1, s1, q2, s2, k=1, group_size=0, act_dtype=oracle.F16,
                             finished=np.ones(T, dtype=np.uint8))
    assert not every["out"].any() and not every["expert_offsets"].any()
    assert np.array_equal(every["perm_src"], np.arange(T))


def test_combine_ignores_pruned_rows_even_if_they_hold_garbage():
    rng = np.random.default_rng(4)
    T, k, d = 6, 2, 8
    y = rng.standard_normal((T * k, d)).astype(np.float32)
    inv = rng.permutation(T * k).astype(np.int32)
    scale = rng.random((T, k)).astype(np.float32)
    active = 7
    y_bad = y.copy()
    y_bad[active:] = np.nan
    got = oracle.combine(y_bad, inv, scale, T, k, active_rows=active)
    want = np.zeros((T, d))
    for t in range(T):
        for j in range(k):
            r = inv[t * k + j]
            if r < active:
                want[t] += float(scale[t, j]) * y[r].astype(np.float64)
    assert np.allclose(got, want, rtol=1e-6, atol=1e-7) and np.isfinite(got).all()
