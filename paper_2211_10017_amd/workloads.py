"""Seeded synthetic inputs for the MoE expert-layer workloads.

This module only draws random numbers and casts them; it holds none of the layer's
arithmetic (no gating, quantisation, routing or matmul) and is the one module that both the
HIP path's callers and the CPU oracle's callers use, so both see the same inputs.

The shapes follow the paper's model (d_model 1024, d_ff 4096, 32 experts, ~40 decoder tokens
per step: Sec. 3.1 and the caption of Table 1) and the benchmark configurations built on it.
The paper's own evaluation data (WMT sentences) is not used; these inputs stand in for it.

Every tensor comes from its own Philox stream ``key=[seed, stream]`` so that experts can be
generated one at a time (the largest configuration's fp32 masters are 34 GB in total).
Real tensors are returned as float32 numpy arrays whose values are exactly representable in
the storage dtype named by the workload ("f16" or "bf16").
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np
import torch

_STREAM_X, _STREAM_WG, _STREAM_BIAS, _STREAM_W1, _STREAM_W2 = 0, 1, 2, 1000, 2000

_TORCH_DTYPE = {"f16": torch.float16, "bf16": torch.bfloat16, "f32": torch.float32}


@dataclass(frozen=True)
class Workload:
    name: str
    T: int              # tokens
    d: int              # d_model
    F: int              # d_ff
    E: int              # experts
    k: int              # experts per token
    bits: int           # 4 or 8
    group_size: int     # 0 = one scale per output channel; else rows of K per scale
    seed: int
    act: str = "f16"    # storage dtype of activations
    bias_kind: str = "none"     # "none" | "uniform" | "zipf"
    bias_param: float = 0.0     # half-width a of U(-a, a) / multiplier c of the Zipf log-weights
    dead_experts: int = 0       # zipf only: experts whose bias is forced to -30 (never chosen)
    renormalize: bool = True
    w_std: float = 0.02

    @property
    def R(self) -> int:
        return self.T * self.k


# bias_param values were chosen once so that the routed loads have the statistics the
# configurations ask for (checked in tests/test_workloads.py):
#   c3: expert loads spread roughly 2x around the mean; c4: the 8 busiest experts receive
#   about 40 % of the assignments and some experts receive none.
WORKLOADS = {
    "c1": Workload("c1", T=256, d=512, F=2048, E=8, k=1, bits=8, group_size=0, seed=0),
    "c2": Workload("c2", T=64, d=1024, F=4096, E=32, k=2, bits=4, group_size=0, seed=1),
    "c3": Workload("c3", T=16384, d=1024, F=4096, E=64, k=1, bits=4, group_size=0, seed=2,
                   bias_kind="uniform", bias_param=0.18),
    "c4": Workload("c4", T=4096, d=2048, F=8192, E=128, k=2, bits=8, group_size=0, seed=3,
                   bias_kind="zipf", bias_param=0.09, dead_experts=6),
    "c5": Workload("c5", T=8192, d=4096, F=16384, E=64, k=2, bits=4, group_size=128, seed=4),
    "c5_bf16": Workload("c5_bf16", T=8192, d=4096, F=16384, E=64, k=2, bits=4, group_size=128,
                        seed=4, act="bf16"),
}


def scaled(w: Workload, **kw) -> Workload:
    """A smaller (or otherwise altered) copy of a workload, e.g. for CPU-sized parity cases."""
    return replace(w, **kw)


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed, stream]))


def cast_to(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round float32 values to the storage dtype (library cast) and return them as float32."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.to(_TORCH_DTYPE[dtype]).to(torch.float32).numpy()


def activations(w: Workload) -> np.ndarray:
    """x [T, d] ~ N(0, 1), rounded to the activation dtype."""
    x = _rng(w.seed, _STREAM_X).standard_normal((w.T, w.d), dtype=np.float32)
    return cast_to(x, w.act)


def gate_weight(w: Workload) -> np.ndarray:
    """Wg [d, E] ~ N(0, 0.02), rounded to the activation dtype."""
    g = _rng(w.seed, _STREAM_WG).standard_normal((w.d, w.E), dtype=np.float32) * np.float32(w.w_std)
    return cast_to(g, w.act)


def gate_bias(w: Workload):
    """Per-expert router bias [E] float32, or None."""
    rng = _rng(w.seed, _STREAM_BIAS)
    if w.bias_kind == "none":
        return None
    if w.bias_kind == "uniform":
        return rng.uniform(-w.bias_param, w.bias_param, w.E).astype(np.float32)
    if w.bias_kind == "zipf":
        # popularity z_e ~ Zipf(s=1.2), bias = c * ln z_e; the `dead_experts` least popular
        # experts (smallest draw, ties by index) are switched off so that they stay empty
        z = rng.zipf(1.2, w.E).astype(np.float64)
        b = (w.bias_param * np.log(z)).astype(np.float32)
        order = np.lexsort((np.arange(w.E), z))
        b[order[:w.dead_experts]] = np.float32(-30.0)
        return b
    raise ValueError(w.bias_kind)


def expert_weight(w: Workload, which: int, e: int) -> np.ndarray:
    """fp32 master of one expert matrix: which=1 -> W1[e] [d, F]; which=2 -> W2[e] [F, d]."""
    shape = (w.d, w.F) if which == 1 else (w.F, w.d)
    stream = (_STREAM_W1 if which == 1 else _STREAM_W2) + e
    a = _rng(w.seed, stream).standard_normal(shape, dtype=np.float32)
    a *= np.float32(w.w_std)
    return a


def expert_weight_batches(w: Workload, which: int, batch: int = 8, threads: int = 8):
    """Yields (first_expert, [masters...]) for consecutive experts, drawn by a thread pool
    (each expert has its own stream, so the result does not depend on the batching)."""
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=threads) as pool:
        for e0 in range(0, w.E, batch):
            es = list(range(e0, min(e0 + batch, w.E)))
            yield e0, list(pool.map(lambda e: expert_weight(w, which, e), es))


def expert_weights(w: Workload, which: int) -> np.ndarray:
    """All experts of one matrix, [E, K, N] float32 (use only when it fits in host memory)."""
    return np.stack([expert_weight(w, which, e) for e in range(w.E)])
