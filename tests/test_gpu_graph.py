"""The decode-sized layer step recorded into a HIP graph (stream capture through torch) and replayed: every
replay, with other work and synchronisations between the replays, must give the bits of the eager call.
The library enqueues kernel launches only (no memset or copy nodes, no allocation), which is what makes the
sequence recordable."""
import numpy as np
import pytest
import torch

from helpers import to_dev
from paper_2211_10017_amd import MoEExpertLayer
from paper_2211_10017_amd import binding as B

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("T,k,E,d,F,bits", [(64, 2, 32, 1024, 1024, 4),      # the decode kernel and its slice reduction
                                            (48, 2, 16, 256, 512, 8)])       # gate, permute, streaming FFN, combine
def test_layer_step_replays_from_a_graph(T, k, E, d, F, bits):
    print(f"graph replay T={T} k={k} E={E} d={d} F={F} bits={bits}", flush=True)
    rng = np.random.default_rng(5 + T)
    layer = MoEExpertLayer(T, d, F, E, k, bits)
    for e in range(E):
        layer.load_expert(1, e, to_dev((rng.standard_normal((d, F)) * 0.05).astype(np.float32), torch.float32))
        layer.load_expert(2, e, to_dev((rng.standard_normal((F, d)) * 0.05).astype(np.float32), torch.float32))
    layer.wg.copy_(to_dev(rng.standard_normal((d, E)).astype(np.float32), torch.float16))
    x = torch.empty((T, d), dtype=torch.float16, device="cuda:0")         # the graph's input buffer
    inputs = [to_dev(rng.standard_normal((T, d)).astype(np.float32), torch.float16) for _ in range(3)]
    eager = []
    for xi in inputs:
        x.copy_(xi)
        eager.append(layer.forward(x).clone())
    torch.cuda.synchronize()
    kernels = B.load().moe_last_ffn_kernels().decode()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        layer.forward(x)
    torch.cuda.synchronize()
    for rep in range(2):
        for xi, want in zip(inputs, eager):
            x.copy_(xi)
            layer.out.fill_(7.0)                                         # eager work of the program's own between replays
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(layer.out, want), f"replay differs from the eager call ({kernels})"
    print(f"   6 replays bit-identical to the eager calls ({kernels})", flush=True)
