"""Parity at the benchmark's full sizes, in the launch configuration bench.py
times: routing and dispatch on every token and every send-buffer row; outputs
on every token where the oracle does the whole batch in seconds, otherwise on
at least 2048 (65 536-token step: 4096) tokens that include, for every local
expert, the rows around every possible M-tile border; plus properties that
hold at any size."""
import numpy as np
import pytest
import torch

from workloads import gen
from helpers import (TOL, border_tokens, check_dispatch, check_routing, dev, host, inputs,
                     make_layer, oracle_out_for_tokens, oracle_route, rel_err)

pytestmark = pytest.mark.gpu

# tokens the output is compared on: None = all of them
OUT_TOKENS = {"c2d": None, "c2p": None, "c3d": None, "c3": None, "c5": None,
              "c4": 2048, "c4w": 2048, "c4q": 2048, "c2x": 4096}


@pytest.mark.parametrize("name", ["c2d", "c2p", "c3d", "c3", "c5", "c4", "c4w", "c4q", "c2x"])
def test_full_size_workload(name):
    w = gen.CONFIGS[name]
    print("workload", name, "generating inputs", flush=True)
    d = inputs(w)
    L = make_layer(w, d)
    x = dev(d["x"])
    forced = None if d["forced"] is None else (dev(d["forced"][0]), dev(d["forced"][1]))
    out = host(L.forward(x, forced)).copy()
    torch.cuda.synchronize()
    print("gpu done; oracle routing", flush=True)
    if forced is None:
        ids_ref, w_ref, margin = oracle_route(w, d["x"], d["gate"])
        n_amb = check_routing(host(L.topk_ids), host(L.topk_w), ids_ref, w_ref, margin,
                              w.routed_scale, name)
        print("fp64-ambiguous tokens:", n_amb, flush=True)
    else:
        ids_ref, w_ref = d["forced"]
    counts, offsets, perm, inv = check_dispatch(L, ids_ref, w, d["x"])
    assert counts.sum() == offsets[-1] <= w.T * w.k
    print("dispatch exact on every row; A_loc =", int(offsets[-1]), "max/min count", counts.max(),
          counts.min(), flush=True)

    iv = inv.reshape(w.T, w.k)
    if OUT_TOKENS[name] is None:
        tokens = np.arange(w.T)
    else:
        tokens = border_tokens(w, offsets, perm, OUT_TOKENS[name])
    print("oracle on %d tokens" % len(tokens), flush=True)
    ref = oracle_out_for_tokens(w, d, tokens, ids_ref, w_ref)
    err = rel_err(out[tokens], ref)
    print("%d tokens: max|err|/max|ref| = %.3e" % (len(tokens), err), flush=True)
    assert err <= TOL[w.weight_dtype], err

    # properties at any size
    if not w.shared_expert:
        none_local = ~(iv >= 0).any(axis=1)
        assert np.all(out[none_local] == 0)
    assert np.isfinite(out).all()
    out2 = host(L.forward(x, forced))
    torch.cuda.synchronize()
    assert np.array_equal(out, out2), "the path is not deterministic"
