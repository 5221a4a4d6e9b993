"""Parity at the benchmark's full sizes, in the launch configuration bench.py
times: routing and dispatch on every token, outputs on sampled tokens the
oracle computes one by one, plus properties that hold at any size."""
import numpy as np
import pytest
import torch

from workloads import gen
from helpers import (TOL, check_dispatch, check_routing, dev, host, inputs, make_layer,
                     oracle_out_for_tokens, oracle_route, rel_err)

pytestmark = pytest.mark.gpu


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
        n_re = int(L.ws[:4].view(torch.int32).item()) if False else None
        print("fp64-ambiguous tokens:", n_amb, flush=True)
    else:
        ids_ref, w_ref = d["forced"]
    counts, offsets, perm, inv = check_dispatch(L, ids_ref, w, d["x"])
    assert counts.sum() == offsets[-1] <= w.T * w.k
    print("dispatch exact; A_loc =", int(offsets[-1]), "max/min count", counts.max(), counts.min(),
          flush=True)

    # sampled tokens: random ones, plus tokens of the most and least loaded experts
    rng = np.random.default_rng(7)
    pick = set(rng.integers(0, w.T, 24).tolist())
    iv = inv.reshape(w.T, w.k)
    for e in (int(np.argmax(counts)), int(np.argmin(np.where(counts > 0, counts, 1 << 30)))):
        rows = perm[offsets[e]:offsets[e + 1]]
        pick.update((rows[:4] // w.k).tolist())
        pick.update((rows[-4:] // w.k).tolist())
    tokens = np.array(sorted(pick))
    ref = oracle_out_for_tokens(w, d, tokens, ids_ref, w_ref)
    err = rel_err(out[tokens], ref)
    print("sampled %d tokens: max|err|/max|ref| = %.3e" % (len(tokens), err), flush=True)
    assert err <= TOL[w.weight_dtype], err

    # properties at any size
    if not w.shared_expert:
        none_local = ~(iv >= 0).any(axis=1)
        assert np.all(out[none_local] == 0)
    assert np.isfinite(out).all()
    out2 = host(L.forward(x, forced))
    torch.cuda.synchronize()
    assert np.array_equal(out, out2), "the path is not deterministic"
