"""The whole pass recorded into a HIP graph: every replay must give what the
eager launches give on the same inputs, also after new data has been copied
into the input buffer and with eager work between the replays."""
import numpy as np
import pytest
import torch

from workloads import gen
from helpers import dev, host, inputs, make_layer

pytestmark = pytest.mark.gpu

CASES = {
    # decode-sized full layer: launch-bound, the case graphs are for
    "decode": gen.CONFIGS["c2d"].replace(name="graph_decode", T=64, H=512, E=32, k=4, I=256),
    # prefill-sized groups (256-row kernel)
    "prefill": gen.CONFIGS["c2p"].replace(name="graph_prefill", T=1024, H=512, E=8, k=2, I=256),
    # enough tokens for the tiled gate GEMM, the interval test with its re-scoring list
    # (a counter cleared by a kernel inside the graph) and the multi-kernel dispatch
    "tiled_route": gen.CONFIGS["c3"].replace(name="graph_tiled", T=4500, H=512, E=128, k=8, I=64,
                                             expert_lo=0, expert_hi=4),
    # shared expert on its second stream inside the capture, sigmoid grouped routing
    "shared": gen.CONFIGS["c4"].replace(name="graph_shared", T=300, H=512, E=64, k=8, I=256,
                                        expert_lo=0, expert_hi=16),
    # e4m3 weights with enough rows per expert for the tall-tile kernel's fp8 weight tiles
    "fp8_weights": gen.CONFIGS["c5"].replace(name="graph_fp8", T=300, H=512, E=64, k=8, I=256,
                                             expert_lo=0, expert_hi=16, zipf_s=None),
    # long gate rows at a few tokens: the exact route as two kernels
    "long_gate_rows": gen.CONFIGS["c3"].replace(name="graph_long_rows", T=9, H=8192, E=128, k=8, I=64,
                                                expert_lo=0, expert_hi=16),
}


@pytest.mark.parametrize("name", list(CASES))
def test_graph_replays_match_eager(name):
    w = CASES[name]
    d = inputs(w)
    L = make_layer(w, d)
    x_np = d["x"]
    rng = np.random.default_rng(5)
    variants = [x_np, x_np[rng.permutation(w.T)], x_np[::-1].copy()]
    x = dev(x_np).clone()
    eager = []
    for v in variants:
        x.copy_(dev(v))
        out = L.forward(x)
        torch.cuda.synchronize()
        eager.append((host(out).copy(), host(L.topk_ids).copy(), host(L.inv).copy()))
    x.copy_(dev(variants[0]))
    graph = L.capture(x)
    for rep in range(2):
        for v, (out_e, ids_e, inv_e) in zip(variants, eager):
            x.copy_(dev(v))
            L.out.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            assert np.array_equal(host(L.topk_ids), ids_e)
            assert np.array_equal(host(L.inv), inv_e)
            assert np.array_equal(host(L.out), out_e), "replay differs from the eager pass"
            # eager work between replays
            L.forward(x)
            torch.cuda.synchronize()
            assert np.array_equal(host(L.out), out_e)
