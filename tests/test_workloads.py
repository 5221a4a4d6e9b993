"""The seeded input generator: determinism, shapes, value distributions."""
import numpy as np

import oracle
from workloads import gen


def test_streams_are_independent_and_reproducible():
    w = gen.CONFIGS["c1"]
    a = gen.make_x(w)
    g = gen.make_gate(w)
    b = gen.make_x(w)
    assert np.array_equal(a, b) and a.dtype == np.float32 and a.shape == (64, 256)
    e1 = gen.make_expert_weights(w, [3])
    e2 = gen.make_expert_weights(w, [0, 3])
    assert np.array_equal(e1["w_gate"][0], e2["w_gate"][1])
    assert e1["w_gate"].shape == (1, 512, 256) and e1["w_down"].shape == (1, 256, 512)
    assert abs(a.std() - 0.02) < 1e-3 and abs(g["gate_w"].std() - 1 / 16) < 3e-3


def test_bf16_gate_logits_are_unit_normal():
    w = gen.CONFIGS["c2d"].replace(T=256)
    x = oracle.decode(gen.make_x(w)).astype(np.float64)
    gw = oracle.decode(gen.make_gate(w)["gate_w"]).astype(np.float64)
    z = x @ gw.T
    assert abs(z.mean()) < 0.02 and abs(z.std() - 1.0) < 0.02


def test_tp_slices_differ_and_fp8_shapes():
    w = gen.CONFIGS["c5"].replace(H=256, I=512, E=16, expert_hi=2)
    a = gen.make_local_experts(w, tp_rank=0)
    b = gen.make_local_experts(w, tp_rank=1)
    assert a["w_gate"].dtype == np.uint8 and a["w_gate"].shape == (2, 256, 256)
    assert a["s_gate"].shape == (2, 2, 2) and a["s_down"].shape == (2, 2, 2)
    assert not np.array_equal(a["w_gate"], b["w_gate"])
    sh = gen.make_shared_expert(w)
    assert sh["w_up"].shape == (1, 256, 256)


def test_forced_zipf_routing():
    w = gen.CONFIGS["c5"]
    ids, wts = gen.make_forced_routing(w)
    ids2, _ = gen.make_forced_routing(w)
    assert np.array_equal(ids, ids2)
    assert ids.shape == (256, 8) and ids.min() >= 0 and ids.max() < 256
    assert all(len(set(r)) == 8 for r in ids)
    np.testing.assert_allclose(wts.sum(1), 2.5, rtol=1e-6)
    cnt = np.bincount(ids.ravel(), minlength=256)
    assert cnt.sum() == 256 * 8
    hottest = np.argsort(-cnt)[:5]
    assert cnt[hottest[0]] > 0.8 * 256                 # the rank-1 expert is in most tokens
    # the stress is only real if hot experts are local to this GPU
    assert np.sum((hottest >= w.expert_lo) & (hottest < w.e_hi)) >= 2
