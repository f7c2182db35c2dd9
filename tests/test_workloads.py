"""The synthetic inputs have the shapes, dtypes and routed-load statistics the benchmark
configurations describe (the load statistics are measured with the oracle's gate)."""
import numpy as np
import pytest

import oracle
from paper_2211_10017_amd import workloads as W


def _loads(w):
    idx, _ = oracle.gate(W.activations(w), W.gate_weight(w), W.gate_bias(w), w.k, w.renormalize)
    return np.bincount(idx.ravel(), minlength=w.E)


def test_shapes_dtypes_and_determinism():
    w = W.WORKLOADS["c2"]
    x, wg = W.activations(w), W.gate_weight(w)
    assert x.shape == (64, 1024) and wg.shape == (1024, 32) and x.dtype == np.float32
    assert np.array_equal(x, x.astype(np.float16).astype(np.float32))        # fp16-representable
    assert abs(float(x.std()) - 1.0) < 0.02 and abs(float(wg.std()) - 0.02) < 0.002
    assert np.array_equal(W.activations(w), x)
    w1 = W.expert_weight(w, 1, 3)
    assert w1.shape == (1024, 4096) and abs(float(w1.std()) - 0.02) < 1e-3
    assert np.array_equal(w1, W.expert_weight(w, 1, 3)) and not np.array_equal(w1[:, :1024], W.expert_weight(w, 2, 3)[:1024])
    xb = W.activations(W.WORKLOADS["c5_bf16"])[:64]
    assert np.array_equal(xb.view(np.uint32) & 0xffff, np.zeros_like(xb, dtype=np.uint32))


def test_c3_loads_vary_about_2x_around_the_mean():
    cnt = _loads(W.WORKLOADS["c3"])
    mean = cnt.mean()
    assert cnt.sum() == 16384 and cnt.min() > 0
    assert 1.6 < cnt.max() / mean < 2.4 and 0.25 < cnt.min() / mean < 0.7


def test_c4_is_skewed_with_empty_experts():
    cnt = _loads(W.WORKLOADS["c4"])
    assert cnt.sum() == 8192
    top8 = np.sort(cnt)[-8:].sum() / cnt.sum()
    assert 0.35 < top8 < 0.45 and (cnt == 0).sum() >= 1


@pytest.mark.parametrize("name,rows", [("c1", 256), ("c2", 128)])
def test_small_configs_route_every_assignment(name, rows):
    cnt = _loads(W.WORKLOADS[name])
    assert cnt.sum() == rows
