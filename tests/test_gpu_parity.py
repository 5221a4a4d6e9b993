"""HIP path vs CPU oracle through the C ABI, element by element, on small and
scaled-down workloads that still span several tiles and ragged tails."""
import numpy as np
import pytest
import torch

import oracle
from workloads import gen
from helpers import (TOL, check_dispatch, check_routing, dev, host, inputs, make_layer,
                     oracle_out_for_tokens, oracle_route, rel_err)

pytestmark = pytest.mark.gpu

SMALL = {
    "c1": gen.CONFIGS["c1"],
    # Qwen3-like, ragged T, several M tiles per expert for some experts
    "qwen_small": gen.CONFIGS["c2p"].replace(name="qwen_small", T=777, H=512, E=32, k=4, I=384),
    # EP share with skew bias
    "ep_small": gen.CONFIGS["c3"].replace(name="ep_small", T=1500, H=256, E=64, k=8, I=256,
                                          expert_lo=8, expert_hi=16),
    # DeepSeek-like: sigmoid, groups, shared expert, TP slice
    "ds_small": gen.CONFIGS["c4"].replace(name="ds_small", T=1111, H=512, E=64, k=8, I=512,
                                          expert_lo=16, expert_hi=24),
    # decode-like: few tokens per expert
    "decode_small": gen.CONFIGS["c2d"].replace(name="decode_small", T=19, H=512, E=32, k=4, I=256),
    # medium rows per expert (the 64-row M tile)
    "mid_small": gen.CONFIGS["c2p"].replace(name="mid_small", T=100, H=256, E=16, k=8, I=128),
    # fp8 weights, few rows per expert (short M tiles), no group limit
    "fp8_decode_small": gen.CONFIGS["c5"].replace(name="fp8_decode_small", T=40, H=256, E=16, k=4,
                                                  I=256, expert_lo=0, expert_hi=16, zipf_s=None,
                                                  n_groups=1, topk_groups=1, group_score_n=0),
    # sizes that are not multiples of the tile shapes: K and N tails, odd E and k
    "ragged_dims": gen.CONFIGS["c2p"].replace(name="ragged_dims", T=333, H=328, E=20, k=3, I=200),
    "ragged_dims_decode": gen.CONFIGS["c2d"].replace(name="ragged_dims_decode", T=9, H=136, E=12,
                                                     k=5, I=72),
    # prefill-size groups whose K is not a multiple of 64 (generic 128-row kernel)
    "ragged_dims_prefill": gen.CONFIGS["c2p"].replace(name="ragged_dims_prefill", T=900, H=328, E=4,
                                                      k=2, I=200),
    # prefill-size groups on the 256-row kernel with N tails (I = 128+64, H = 256+64)
    "tail_256": gen.CONFIGS["c2p"].replace(name="tail_256", T=900, H=320, E=4, k=2, I=192),
    # many experts per lane slot and a large k
    "wide_gate": gen.CONFIGS["c2p"].replace(name="wide_gate", T=150, H=256, E=512, k=16, I=64,
                                            expert_lo=100, expert_hi=400),
    # rows shorter than a wavefront's 64 pieces, and rows whose last pieces are a second,
    # partly filled pass of the wavefront (the combine walks a row in 64-piece steps)
    "hidden_8": gen.CONFIGS["c2p"].replace(name="hidden_8", T=40, H=8, E=16, k=3, I=704, tp=2,
                                           shared_expert=True, expert_lo=10, expert_hi=12),
    "f32_hidden_264": gen.CONFIGS["c1"].replace(name="f32_hidden_264", T=2500, H=264, E=32, k=3,
                                                I=80, tp=2, expert_lo=30, expert_hi=31),
    # fp8 weights, natural routing
    "fp8_small": gen.CONFIGS["c5"].replace(name="fp8_small", T=300, H=512, E=64, k=8, I=512,
                                           expert_lo=0, expert_hi=8, zipf_s=None),
}


def run_full(w):
    d = inputs(w)
    L = make_layer(w, d)
    x = dev(d["x"])
    forced = None
    if d["forced"] is not None:
        forced = (dev(d["forced"][0]), dev(d["forced"][1]))
    out = L.forward(x, forced)
    torch.cuda.synchronize()
    return d, L, host(out)


@pytest.mark.parametrize("name", list(SMALL))
def test_layer_share_matches_oracle(name):
    w = SMALL[name]
    print("case", name, flush=True)
    d, L, out = run_full(w)
    ids_ref, w_ref, margin = oracle_route(w, d["x"], d["gate"])
    ids, wts = host(L.topk_ids), host(L.topk_w)
    check_routing(ids, wts, ids_ref, w_ref, margin, w.routed_scale, name)
    check_dispatch(L, ids_ref, w, d["x"])
    ref, parts = oracle.layer_share(d["x"], ids_ref, w_ref, w.expert_lo, w.e_hi, d["experts"],
                                    d["shared"])
    n = int(parts["offsets"][-1])
    ys = oracle.decode(host(L.ys[:n])) if w.act_dtype == "bf16" else host(L.ys[:n])
    tol = TOL[w.weight_dtype]
    assert n == 0 or rel_err(ys, parts["ys"][:n]) <= tol
    assert rel_err(out, ref) <= tol, rel_err(out, ref)


def test_route_recheck_counter_and_determinism():
    w = SMALL["qwen_small"]
    d = inputs(w)
    L = make_layer(w, d)
    x = dev(d["x"])
    L.route(x)
    torch.cuda.synchronize()
    n1 = int(L.ws[:4].view(torch.int32).item())
    a = (host(L.topk_ids).copy(), host(L.topk_w).copy())
    L.route(x)
    torch.cuda.synchronize()
    assert int(L.ws[:4].view(torch.int32).item()) == n1 and 0 <= n1 <= w.T
    assert np.array_equal(a[0], host(L.topk_ids)) and np.array_equal(a[1], host(L.topk_w))


# Token counts past the decode-size threshold of the router (T*E*H > 2^28, or more
# than 4096 tokens), so the
# tiled bf16 gate GEMM, the interval test and the fp64 re-scoring run, at sizes
# the oracle still scores in seconds: ragged T / E / H tails, with and without a
# split K range, soft-max with a logit bias and sigmoid with a group limit.
TILED_GATE = {
    "softmax_ragged_splitk": gen.CONFIGS["c2p"].replace(name="softmax_ragged_splitk", T=1237, H=1096,
                                                        E=200, k=6, I=64),
    "softmax_bias_one_slab": gen.CONFIGS["c3"].replace(name="softmax_bias_one_slab", T=4500, H=512,
                                                       E=128, k=8, I=64, expert_lo=0, expert_hi=4),
    # many token tiles, ragged T and E, one K slab
    "tall_tile_ragged": gen.CONFIGS["c2p"].replace(name="tall_tile_ragged", T=8300, H=512, E=72, k=4,
                                                   I=64),
    # fp32 activations past the one-kernel route: fp64 VALU gate, then select / re-score
    "f32_many_tokens": gen.CONFIGS["c1"].replace(name="f32_many_tokens", T=4200, H=256, E=16, k=2,
                                                 I=64),
    "sigmoid_groups_splitk": gen.CONFIGS["c4"].replace(name="sigmoid_groups_splitk", T=2100, H=1024,
                                                       E=192, k=6, I=128, n_groups=6, topk_groups=3,
                                                       expert_lo=0, expert_hi=8),
}


# The same pipeline at up to 1024 tokens, where the re-scoring kernel gives a listed
# token a whole workgroup (its wavefronts share each dot product).
TILED_GATE.update({
    "short_list_softmax": gen.CONFIGS["c2p"].replace(name="short_list_softmax", T=777, I=64),
    "short_list_softmax_1024": gen.CONFIGS["c3"].replace(name="short_list_softmax_1024", T=1024, I=64,
                                                         expert_lo=0, expert_hi=4),
    "short_list_sigmoid_groups": gen.CONFIGS["c4"].replace(name="short_list_sigmoid_groups", T=301,
                                                           I=128, shared_expert=False),
    "short_list_f32": gen.CONFIGS["c1"].replace(name="short_list_f32", T=1000, H=2048, E=160, k=4,
                                                I=64),
})


@pytest.mark.parametrize("name", list(TILED_GATE))
def test_route_tiled_gate_matches_oracle(name):
    w = TILED_GATE[name]
    assert w.T * w.E * w.H > 2 ** 28 or w.T > 4096 or (w.act_dtype == "bf16" and w.T * w.E * w.H > 5 * 2 ** 25)
    print("case", name, flush=True)
    d = inputs(w)
    L = make_layer(w, d)
    L.route(dev(d["x"]))
    torch.cuda.synchronize()
    n_re = int(L.ws[:4].view(torch.int32).item())
    ids_ref, w_ref, margin = oracle_route(w, d["x"], d["gate"])
    n_amb = check_routing(host(L.topk_ids), host(L.topk_w), ids_ref, w_ref, margin,
                          w.routed_scale, name)
    print("re-scored", n_re, "of", w.T, "; fp64-ambiguous", n_amb, flush=True)
    assert 0 <= n_re <= w.T


# Few tokens, long gate rows (E*H > 2^19): exact logits and selection run as two
# kernels, a token's experts shared out over several workgroups.  Group-limited
# sigmoid at the C4 gate shape, soft-max with 512 and with an odd number of
# experts, fp32 inputs; one token, and token counts that are no multiple of four.
LONG_ROWS = {
    "c4_gate_1_token": gen.CONFIGS["c4"].replace(name="c4_gate_1_token", T=1, I=128, shared_expert=False),
    "c4_gate_67_tokens": gen.CONFIGS["c4"].replace(name="c4_gate_67_tokens", T=67, I=128,
                                                   shared_expert=False),
    "softmax_512_experts": gen.CONFIGS["c3"].replace(name="softmax_512_experts", T=130, E=512, H=2048,
                                                     I=64, expert_lo=0, expert_hi=8),
    "softmax_130_experts": gen.CONFIGS["c3"].replace(name="softmax_130_experts", T=5, E=130, H=8192,
                                                     I=64, expert_lo=0, expert_hi=8),
    "f32_72_experts": gen.CONFIGS["c1"].replace(name="f32_72_experts", T=130, E=72, H=8192, I=64, k=4),
}


@pytest.mark.parametrize("name", list(LONG_ROWS))
def test_route_long_gate_rows_matches_oracle(name):
    w = LONG_ROWS[name]
    assert w.E * w.H > 2 ** 19 and w.T * w.E * w.H <= 2 ** 28
    print("case", name, flush=True)
    x, gate = gen.make_x(w), gen.make_gate(w)
    L = make_layer(w, {"gate": gate, "experts": gen.make_local_experts(w), "shared": None})
    L.route(dev(x))
    torch.cuda.synchronize()
    assert int(L.ws[:4].view(torch.int32).item()) == 0          # exact keys: nothing to re-score
    ids_ref, w_ref, margin = oracle_route(w, x, gate)
    check_routing(host(L.topk_ids), host(L.topk_w), ids_ref, w_ref, margin, w.routed_scale, name)


@pytest.mark.parametrize("E,k,score,G,Kg,gn", [
    (8, 2, "softmax", 1, 1, 0), (64, 6, "softmax", 1, 1, 0), (100, 8, "softmax", 1, 1, 0),
    (128, 8, "softmax", 1, 1, 0), (256, 8, "sigmoid", 8, 4, 2), (256, 8, "sigmoid", 1, 1, 0),
    (96, 4, "sigmoid", 6, 3, 1), (512, 32, "softmax", 1, 1, 0), (48, 5, "sigmoid", 4, 2, 3)])
def test_selection_logic_on_given_logits(E, k, score, G, Kg, gn):
    """Identical fp32 logits on both sides: the selection alone must be bit-exact."""
    from paper_2601_08800_amd import MoELayerShare
    from paper_2601_08800_amd.layer import config_from_workload
    T = 513
    rng = np.random.default_rng(E * 7 + k)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    logits[5] = 0.25                       # a row of exact ties
    logits[6, : E // 2] = 1.0              # partial ties
    w = gen.CONFIGS["c2d"].replace(T=T, H=64, E=E, k=k, I=64, score_fn=score, n_groups=G,
                                   topk_groups=Kg, group_score_n=gn, routed_scale=2.5,
                                   select_bias_std=0.05 if score == "sigmoid" else 0.0,
                                   logit_bias_std=0.3 if score == "softmax" else 0.0)
    gate = gen.make_gate(w)
    ids_ref, w_ref, margin = oracle_route(w, None, gate, logits_in=logits)
    L = MoELayerShare(config_from_workload(w), T, gate,
                      {"w_gate": None, "w_up": None, "w_down": None})
    L.route(None, logits_in=dev(logits))
    torch.cuda.synchronize()
    ids, wts = host(L.topk_ids), host(L.topk_w)
    assert np.array_equal(ids, ids_ref)
    np.testing.assert_allclose(wts, w_ref, rtol=2e-5, atol=5e-6)


def test_exact_arithmetic_gate_with_ties():
    """Small-integer activations and gate weights: every summation order gives
    the same logits, so ids must match exactly, deliberate ties included."""
    from paper_2601_08800_amd import MoELayerShare
    from paper_2601_08800_amd.layer import config_from_workload
    T, H, E, k = 200, 192, 24, 3
    rng = np.random.default_rng(3)
    xi = rng.integers(-3, 4, size=(T, H)).astype(np.float32)
    gi = rng.integers(-2, 3, size=(E, H)).astype(np.float32)
    gi[7] = gi[2]                                             # two identical experts
    for act in ("bf16", "f32"):
        w = gen.CONFIGS["c2d"].replace(T=T, H=H, E=E, k=k, I=64, act_dtype=act,
                                       weight_dtype=act)
        x = gen.f32_to_bf16_bits(xi) if act == "bf16" else xi
        g = gen.f32_to_bf16_bits(gi) if act == "bf16" else gi
        gate = {"gate_w": g, "logit_bias": None, "select_bias": None}
        ids_ref, w_ref, margin = oracle_route(w, x, gate)
        assert (margin == 0).sum() > 0
        L = MoELayerShare(config_from_workload(w), T, gate,
                          {"w_gate": None, "w_up": None, "w_down": None})
        L.route(dev(x))
        torch.cuda.synchronize()
        assert np.array_equal(host(L.topk_ids), ids_ref)
        np.testing.assert_allclose(host(L.topk_w), w_ref, rtol=2e-5)


def test_identity_experts_return_input():
    """Skipping the MLP (ys := xs) the share returns (sum of weights) * x."""
    for name in ("qwen_small", "c1"):
        w = SMALL[name].replace(expert_lo=0, expert_hi=0)
        d = inputs(w)
        L = make_layer(w, d)
        x = dev(d["x"])
        L.route(x)
        L.dispatch(x)
        L.combine(ys=L.xs)
        torch.cuda.synchronize()
        xf = oracle.decode(d["x"])
        assert int(host(L.offsets)[-1]) == w.T * w.k
        assert rel_err(host(L.out), xf) <= (1e-6 if name == "c1" else 2e-6)


@pytest.mark.parametrize("T,e_lo,e_hi", [(1, 0, 16), (3, 5, 6), (1025, 0, 16), (2048, 15, 16),
                                          (64, 3, 9)])
def test_dispatch_edge_cases(T, e_lo, e_hi):
    w = gen.CONFIGS["c2d"].replace(T=T, H=128, E=16, k=4, I=64, expert_lo=e_lo, expert_hi=e_hi)
    rng = np.random.default_rng(T)
    ids = np.stack([rng.permutation(16)[:4] for _ in range(T)]).astype(np.int32)
    if T > 100:
        ids[:, 0] = 15                     # one very hot expert, several empty ones
        ids[:, 1:] = np.stack([rng.permutation(5)[:3] for _ in range(T)])
    d = {"x": gen.make_x(w), "gate": gen.make_gate(w),
         "experts": {"w_gate": None, "w_up": None, "w_down": None}, "shared": None}
    L = make_layer(w, d)
    L.topk_ids = dev(ids)
    L.dispatch(dev(d["x"]))
    torch.cuda.synchronize()
    check_dispatch(L, ids, w, d["x"])


def test_tp_and_ep_additivity_on_gpu():
    """Partial outputs of the TP slices / EP ranges add up to the full layer
    (block matrix multiplication; experts are independent)."""
    base = gen.CONFIGS["c2p"].replace(T=200, H=256, E=16, k=4, I=256)
    d = inputs(base)
    full = make_layer(base, d).forward(dev(d["x"])).clone()
    acc = torch.zeros_like(full)
    for r in range(2):                     # EP = 2
        w = base.replace(expert_lo=8 * r, expert_hi=8 * r + 8)
        acc += make_layer(w, inputs(w)).forward(dev(d["x"]))
    torch.cuda.synchronize()
    assert rel_err(host(acc), host(full)) <= 1e-6
    tp = base.replace(tp=2, I=512)         # two slices of 256
    ids_ref, w_ref, _ = oracle_route(tp, d["x"], d["gate"])
    ref = np.zeros((tp.T, tp.H))
    got = torch.zeros_like(full)
    for r in range(2):
        wr = tp.replace(tp_rank=r)
        dr = inputs(wr)
        got += make_layer(wr, dr).forward(dev(dr["x"]))
        ref += oracle.layer_share(dr["x"], ids_ref, w_ref, 0, 16, dr["experts"])[0]
    torch.cuda.synchronize()
    assert rel_err(host(got), ref) <= TOL["bf16"]


def _forced_counts_case(counts, H=256, I=192, seed=11):
    """One assignment per token (k = 1), expert of token t fixed so that the
    local experts receive exactly `counts` rows, interleaved (not pre-sorted)."""
    E = len(counts)
    T = int(sum(counts))
    ids = np.concatenate([np.full(c, e, np.int32) for e, c in enumerate(counts)])
    ids = ids[np.random.default_rng(seed).permutation(T)].reshape(T, 1)
    tw = (0.5 + np.random.default_rng(seed + 1).random((T, 1))).astype(np.float32)
    w = gen.CONFIGS["c2p"].replace(name="forced_counts", T=T, H=H, E=E, k=1, I=I, seed=4242 + T)
    return w, ids, tw


@pytest.mark.parametrize("counts", [
    [0, 0, 0, 2048, 0, 0, 0, 0],            # one expert takes everything: eight full tiles, seven empty experts
    [256] * 8,                              # every tile full, no tails
    [257, 1, 0, 511, 513, 255, 256, 255],   # one row over / under the tile borders
    [0, 0, 512, 0, 0, 0, 0, 0],             # 64 rows per expert on average, all in one expert
    [0, 64, 0, 0, 0, 0, 0, 0],              # decode-sized, all in one expert
    [1, 0, 0, 0, 0, 0, 0, 0],               # a single row
    [33, 31, 32, 0, 65, 63, 64, 1],         # around the 32-row tiles of the weight-streaming kernel
])
def test_ffn_degenerate_loads(counts):
    """Forced routing with extreme per-expert row counts: every FFN kernel family
    gets empty experts, one hot expert and rows on both sides of its tile borders."""
    w, ids, tw = _forced_counts_case(counts)
    d = inputs(w)
    L = make_layer(w, d)
    out = host(L.forward(dev(d["x"]), (dev(ids), dev(tw))))
    torch.cuda.synchronize()
    c, o, perm, inv = check_dispatch(L, ids, w, d["x"])
    assert c.tolist() == list(counts)
    ref, _ = oracle.layer_share(d["x"], ids, tw, 0, w.E, d["experts"])
    assert rel_err(out, ref) <= TOL["bf16"]
    # rows of ys beyond the last valid one and other experts' rows are untouched by a tile's tail:
    # recompute a few single tokens on their own and compare
    rows = np.unique(np.random.default_rng(3).integers(0, w.T, 8))
    for t in rows:
        one, _ = oracle.layer_share(d["x"][t:t + 1], ids[t:t + 1], tw[t:t + 1], 0, w.E, d["experts"])
        assert rel_err(out[t:t + 1], one) <= TOL["bf16"]


@pytest.mark.parametrize("rows_per_expert", [12, 13])
def test_fp8_weights_on_both_sides_of_the_kernel_switch(rows_per_expert):
    """e4m3 weights: up to twelve rows per expert (rows_capacity / n_experts) the
    weight-streaming kernel applies the block scale to fp32 partial sums, above it
    the tall-tile kernel rounds code * scale to bf16.  Both must meet the fp8
    tolerance against the exact product on the same kind of load."""
    E = 8
    counts = [rows_per_expert] * E
    counts[0] += 5                          # ragged, and one expert above the average
    counts[3] -= 5
    w, ids, tw = _forced_counts_case(counts, H=256, I=256, seed=23)
    w = w.replace(weight_dtype="fp8", name="fp8_switch")
    d = inputs(w)
    L = make_layer(w, d)
    out = host(L.forward(dev(d["x"]), (dev(ids), dev(tw))))
    torch.cuda.synchronize()
    assert w.T // E == rows_per_expert
    check_dispatch(L, ids, w, d["x"])
    ref, _ = oracle.layer_share(d["x"], ids, tw, 0, w.E, d["experts"])
    err = rel_err(out, ref)
    print("rows per expert", rows_per_expert, "err %.3e" % err, flush=True)
    assert err <= TOL["fp8"]


@pytest.mark.parametrize("weight_dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("counts", [[300, 200], [40, 0, 700, 90]])
def test_ffn_k_split_of_leftover_tiles(counts, weight_dtype):
    """Few tiles and a long K (16 K steps in both GEMMs): the tall-tile kernel cuts
    every tile along K into parts whose fp32 partial sums the last part adds up.
    Outputs against the oracle, and twice the same bits."""
    w, ids, tw = _forced_counts_case(counts, H=1024, I=1024, seed=31)
    w = w.replace(weight_dtype=weight_dtype, name="k_split")
    d = inputs(w)
    L = make_layer(w, d)
    x = dev(d["x"])
    out = host(L.forward(x, (dev(ids), dev(tw)))).copy()
    torch.cuda.synchronize()
    check_dispatch(L, ids, w, d["x"])
    ref, _ = oracle.layer_share(d["x"], ids, tw, 0, w.E, d["experts"])
    err = rel_err(out, ref)
    print("counts", counts, weight_dtype, "err %.3e" % err, flush=True)
    assert err <= TOL[weight_dtype]
    for _ in range(3):
        again = host(L.forward(x, (dev(ids), dev(tw))))
        torch.cuda.synchronize()
        assert np.array_equal(out, again), "the sum of the parts depends on their arrival order"


def test_ffn_many_full_tiles_same_bits_every_time():
    """Hundreds of full 256-row tiles with 64 / 16 K steps, more than one round of
    tiles per CU: the form of the K loop in which the two wavefronts of a SIMD run in
    different phases.  A stage of the operand rings refilled while the other row half
    still reads it would show as outputs that change from run to run; outputs
    against the oracle on sampled tokens, and five times the same bits."""
    w, ids, tw = _forced_counts_case([1536] * 8, H=4096, I=1024, seed=57)
    w = w.replace(name="full_tiles")
    d = inputs(w)
    L = make_layer(w, d)
    x = dev(d["x"])
    out = host(L.forward(x, (dev(ids), dev(tw)))).copy()
    torch.cuda.synchronize()
    check_dispatch(L, ids, w, d["x"])
    tokens = np.random.default_rng(3).choice(w.T, 768, replace=False)
    ref = oracle_out_for_tokens(w, d, tokens, ids, tw)
    err = rel_err(out[tokens], ref)
    print("768 tokens: err %.3e" % err, flush=True)
    assert err <= TOL["bf16"]
    for _ in range(5):
        again = host(L.forward(x, (dev(ids), dev(tw))))
        torch.cuda.synchronize()
        assert np.array_equal(out, again), "outputs differ between runs"


@pytest.mark.parametrize("H,I", [(64, 64), (128, 64), (64, 192), (192, 128), (320, 64)])
def test_ffn_full_tiles_short_k(H, I):
    """Full 256-row tiles whose K loops have one to five steps: fewer steps than the
    operand rings have stages, so the alternating form of the loop runs its fill and
    drain paths only (no steady step at all for one and two steps)."""
    w, ids, tw = _forced_counts_case([512, 256, 768], H=H, I=I, seed=23)
    w = w.replace(name="short_k")
    d = inputs(w)
    L = make_layer(w, d)
    x = dev(d["x"])
    out = host(L.forward(x, (dev(ids), dev(tw)))).copy()
    torch.cuda.synchronize()
    check_dispatch(L, ids, w, d["x"])
    ref, _ = oracle.layer_share(d["x"], ids, tw, 0, w.E, d["experts"])
    err = rel_err(out, ref)
    print("H", H, "I", I, "err %.3e" % err, flush=True)
    assert err <= TOL["bf16"]
    again = host(L.forward(x, (dev(ids), dev(tw))))
    torch.cuda.synchronize()
    assert np.array_equal(out, again)


@pytest.mark.parametrize("weight_dtype", ["bf16", "fp8"])
def test_ffn_wide_tiles_of_short_groups(weight_dtype):
    """128 local experts with 0 to 200 rows each (76 on average), hidden 1024 and
    intermediate 512: short groups and enough experts for one 512-weight-row tile per
    CU, so GEMM-2 takes its wide tiles (at most 128 rows x 512 weight rows, all eight
    wavefronts on one row half).  Rows on both sides of the 32-row blocks and of the
    128-row tile height; outputs against the oracle on sampled tokens that include
    every expert's first and last row."""
    rng = np.random.default_rng(77)
    counts = [int(rng.choice([0, 1, 13, 31, 32, 33, 64, 96, 127, 128, 129, 200])) for _ in range(128)]
    w, ids, tw = _forced_counts_case(counts, H=1024, I=512, seed=41)
    w = w.replace(name="wide_tiles", weight_dtype=weight_dtype)
    assert 12 < w.T // 128 <= 128
    d = inputs(w)
    L = make_layer(w, d)
    x = dev(d["x"])
    out = host(L.forward(x, (dev(ids), dev(tw)))).copy()
    torch.cuda.synchronize()
    c, offsets, perm, inv = check_dispatch(L, ids, w, d["x"])
    assert c.tolist() == counts
    edge = [perm[o] for e in range(128) if counts[e] for o in (offsets[e], offsets[e + 1] - 1)]
    tokens = np.unique(np.concatenate([np.asarray(edge, dtype=np.int64),
                                       rng.choice(w.T, 400, replace=False)]))
    ref = oracle_out_for_tokens(w, d, tokens, ids, tw)
    err = rel_err(out[tokens], ref)
    print(weight_dtype, "%d tokens: err %.3e" % (len(tokens), err), flush=True)
    assert err <= TOL[weight_dtype]
    again = host(L.forward(x, (dev(ids), dev(tw))))
    torch.cuda.synchronize()
    assert np.array_equal(out, again)


@pytest.mark.parametrize("weight_dtype", ["bf16", "fp8"])
def test_ffn_k_split_beside_wide_tiles(weight_dtype):
    """64 experts, hidden 3072, intermediate 1024: GEMM-1 (70 row tiles x 8 column
    tiles = 560, 48 more than two rounds of CUs) cuts the 48 leftover tiles along its
    48 K steps into two parts each; GEMM-2 takes its wide tiles."""
    counts = [50] * 64
    for e in (3, 17, 20, 33, 48, 60):
        counts[e] = 200
    w, ids, tw = _forced_counts_case(counts, H=3072, I=1024, seed=5)
    w = w.replace(name="wide_split", weight_dtype=weight_dtype)
    d = inputs(w)
    L = make_layer(w, d)
    x = dev(d["x"])
    out = host(L.forward(x, (dev(ids), dev(tw)))).copy()
    torch.cuda.synchronize()
    c, offsets, perm, inv = check_dispatch(L, ids, w, d["x"])
    edge = [perm[o] for e in range(64) for o in (offsets[e], offsets[e + 1] - 1)]
    tokens = np.unique(np.concatenate([np.asarray(edge, dtype=np.int64),
                                       np.random.default_rng(1).choice(w.T, 300, replace=False)]))
    ref = oracle_out_for_tokens(w, d, tokens, ids, tw)
    err = rel_err(out[tokens], ref)
    print(weight_dtype, "err %.3e" % err, flush=True)
    assert err <= TOL[weight_dtype]
    for _ in range(3):
        again = host(L.forward(x, (dev(ids), dev(tw))))
        torch.cuda.synchronize()
        assert np.array_equal(out, again), "the sum of the parts depends on their arrival order"


def test_ffn_second_tile_table_holds_more_tiles_than_the_first():
    """64 experts alternating 129 rows and one row, hidden 2048, intermediate 512:
    GEMM-2 takes wide tiles (128-row tiles: 96 of them) while GEMM-1 keeps 160-row
    tiles (64), so the second table is the longer one; the last experts' rows are
    the ones a table cut at the first table's bound would lose."""
    counts = [129, 1] * 32
    w, ids, tw = _forced_counts_case(counts, H=2048, I=512, seed=9)
    w = w.replace(name="two_tables")
    d = inputs(w)
    L = make_layer(w, d)
    out = host(L.forward(dev(d["x"]), (dev(ids), dev(tw)))).copy()
    torch.cuda.synchronize()
    c, offsets, perm, inv = check_dispatch(L, ids, w, d["x"])
    edge = [perm[o] for e in range(64) for o in (offsets[e], offsets[e + 1] - 1)]
    tokens = np.unique(np.concatenate([np.asarray(edge, dtype=np.int64), perm[offsets[56]:offsets[64]],
                                       np.random.default_rng(2).choice(w.T, 200, replace=False)]))
    ref = oracle_out_for_tokens(w, d, tokens, ids, tw)
    err = rel_err(out[tokens], ref)
    print("%d tokens: err %.3e" % (len(tokens), err), flush=True)
    assert err <= TOL["bf16"]


def test_ffn_wide_tiles_with_k_split():
    """32 experts, hidden 4096, intermediate 3072: GEMM-2 takes wide tiles (34 row tiles
    x 8 column tiles of 512 = 272, 16 more than the CUs) and cuts the 16 leftover tiles
    along its 48 K steps into two parts each: all eight wavefronts of a part leave
    partial sums, the last part to arrive adds them."""
    counts = [60] * 32
    counts[5] = counts[21] = 200
    w, ids, tw = _forced_counts_case(counts, H=4096, I=3072, seed=6)
    w = w.replace(name="wide_split")
    d = inputs(w)
    L = make_layer(w, d)
    x = dev(d["x"])
    out = host(L.forward(x, (dev(ids), dev(tw)))).copy()
    torch.cuda.synchronize()
    c, offsets, perm, inv = check_dispatch(L, ids, w, d["x"])
    edge = [perm[o] for e in range(32) for o in (offsets[e], offsets[e + 1] - 1)]
    tokens = np.unique(np.concatenate([np.asarray(edge, dtype=np.int64),
                                       np.random.default_rng(1).choice(w.T, 100, replace=False)]))
    ref = oracle_out_for_tokens(w, d, tokens, ids, tw)
    err = rel_err(out[tokens], ref)
    print("err %.3e" % err, flush=True)
    assert err <= TOL["bf16"]
    for _ in range(3):
        again = host(L.forward(x, (dev(ids), dev(tw))))
        torch.cuda.synchronize()
        assert np.array_equal(out, again), "the sum of the parts depends on their arrival order"


def test_mfma_rate_probe_runs_and_is_plausible():
    """The calibration loop of the MFMA roofline: a rate between a tenth of the
    published bf16 peak and the peak itself, and argument validation."""
    import paper_2601_08800_amd as moe
    tf = moe.moe_probe_mfma_rate(512, 500)
    print("register-only MFMA loop: %.0f TFLOP/s" % tf, flush=True)
    assert 250.0 < tf <= 2600.0
    with pytest.raises(moe.MoEError):
        moe.moe_probe_mfma_rate(0, 500)


def _random_workload(seed):
    """A small layer with seeded random shape and gate options (every size a legal
    but awkward one: odd expert counts, k up to 8, ragged token counts, EP ranges)."""
    rng = np.random.default_rng(1000 + seed)
    score = "sigmoid" if rng.random() < 0.5 else "softmax"
    G = 1
    E = int(rng.integers(2, 200))
    if score == "sigmoid" and rng.random() < 0.6:
        G = int(rng.choice([2, 3, 4, 8]))
        E = G * int(rng.integers(2, 24))
    gs = E // G
    Kg = int(rng.integers(1, G + 1)) if G > 1 else 1
    gn = int(rng.integers(1, min(gs, 3) + 1)) if G > 1 else 0
    k = int(rng.integers(1, min(8, Kg * gs if G > 1 else E) + 1))
    lo = int(rng.integers(0, E))
    hi = int(rng.integers(lo + 1, E + 1))
    return gen.CONFIGS["c2p"].replace(
        name="random_%d" % seed, seed=5000 + seed, T=int(rng.integers(1, 400)),
        H=8 * int(rng.integers(8, 64)), E=E, k=k, I=8 * int(rng.integers(4, 24)), score_fn=score,
        renormalize=bool(rng.random() < 0.7), routed_scale=float(rng.choice([1.0, 2.5])),
        n_groups=G, topk_groups=Kg, group_score_n=gn, expert_lo=lo, expert_hi=hi,
        logit_bias_std=float(rng.choice([0.0, 0.5])),
        select_bias_std=0.05 if score == "sigmoid" else 0.0)


@pytest.mark.parametrize("seed", list(range(16)) + [108])     # 108: no token goes to a local expert
def test_random_small_layers(seed):
    w = _random_workload(seed)
    print("case", w, flush=True)
    d, L, out = run_full(w)
    ids_ref, w_ref, margin = oracle_route(w, d["x"], d["gate"])
    check_routing(host(L.topk_ids), host(L.topk_w), ids_ref, w_ref, margin, w.routed_scale, w.name)
    check_dispatch(L, ids_ref, w, d["x"])
    ref, _ = oracle.layer_share(d["x"], ids_ref, w_ref, w.expert_lo, w.e_hi, d["experts"], d["shared"])
    assert rel_err(out, ref) <= TOL["bf16"] or np.abs(ref).max() == 0


def _random_ffn_workload(seed):
    """Seeded random layers that vary what the expert FFN sees: activation / weight
    dtype, shared expert, TP slice, sizes that reach every GEMM family (hidden and
    intermediate sizes that are multiples of 8, 64 or 128; 3 to 2500 tokens)."""
    r = np.random.default_rng(7000 + seed)
    kind = r.choice(["bf16", "fp8", "f32"], p=[0.5, 0.35, 0.15])
    E = int(r.choice([4, 8, 16, 32]))
    k = int(r.integers(1, min(4, E) + 1))
    mult = 128 if kind == "fp8" else (64 if r.random() < 0.5 else 8)
    H = mult * int(r.integers(1, max(2, 1024 // mult)))
    tp = int(r.choice([1, 2]))
    I = tp * mult * int(r.integers(1, max(2, 512 // mult)))
    Tn = int(r.choice([3, 40, 200, 900, 2500]))
    lo = int(r.integers(0, E))
    hi = int(r.integers(lo + 1, E + 1))
    base = gen.CONFIGS["c1"] if kind == "f32" else gen.CONFIGS["c2p"]
    return base.replace(name="random_ffn_%d" % seed, seed=9000 + seed, T=Tn, H=H, E=E, k=k, I=I,
                        expert_lo=lo, expert_hi=hi, tp=tp, tp_rank=int(r.integers(0, tp)),
                        shared_expert=bool(r.random() < 0.4), weight_dtype=str(kind))


# 118 and 183 once exposed the combine's handling of rows shorter than 64 pieces
@pytest.mark.parametrize("seed", [0, 1, 2, 3, 4, 5, 6, 7, 9, 11, 118, 183])
def test_random_ffn_families(seed):
    w = _random_ffn_workload(seed)
    print("case", w, flush=True)
    d, L, out = run_full(w)
    ids_ref, w_ref, margin = oracle_route(w, d["x"], d["gate"])
    check_routing(host(L.topk_ids), host(L.topk_w), ids_ref, w_ref, margin, w.routed_scale, w.name)
    check_dispatch(L, ids_ref, w, d["x"])
    ref, _ = oracle.layer_share(d["x"], ids_ref, w_ref, w.expert_lo, w.e_hi, d["experts"], d["shared"])
    err = rel_err(out, ref) if np.abs(ref).max() > 0 else float(np.abs(out).max())
    assert err <= TOL[w.weight_dtype], err


@pytest.mark.parametrize("seed", range(8))
def test_random_routing_past_4096_tokens(seed):
    """The random gate options of `_random_workload` at 4097..7000 tokens: tiled
    gate GEMM (or the fp64 gate for fp32 inputs), interval test, re-scoring."""
    r = np.random.default_rng(33000 + seed)
    w = _random_workload(seed).replace(T=int(r.integers(4097, 7000)), I=8, name="random_route_%d" % seed)
    if r.random() >= 0.8:
        w = w.replace(act_dtype="f32", weight_dtype="f32")
    print("case", w, flush=True)
    d = inputs(w)
    L = make_layer(w, d)
    L.route(dev(d["x"]))
    torch.cuda.synchronize()
    ids_ref, w_ref, margin = oracle_route(w, d["x"], d["gate"])
    check_routing(host(L.topk_ids), host(L.topk_w), ids_ref, w_ref, margin, w.routed_scale, w.name)
