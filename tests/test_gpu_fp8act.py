"""Expert FFN with 8-bit activations on the GPU against the oracle, through the
C ABI.  The quantisation decisions are fp32 operations on both sides, so the
output of a case whose intermediate rounds the same way matches closely; in
general a bf16-rounding difference in the intermediate can move a code by one
step, which the fp8 tolerance of the layer (6e-2 of the largest reference
value) covers."""
import numpy as np
import pytest
import torch

import oracle
import paper_2601_08800_amd as moe
from paper_2601_08800_amd.layer import config_from_workload
from workloads import gen
from helpers import dev, host, rel_err

pytestmark = pytest.mark.gpu


def run_case(w, counts):
    """Rows of `counts[e]` tokens for local expert e; returns (ys_gpu, ys_ref, n)."""
    cfg = config_from_workload(w)
    n_exp = w.e_hi - w.expert_lo
    assert len(counts) == n_exp
    offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    n = int(offsets[-1])
    cap = max(n, 1) + 37                       # capacity beyond the valid rows
    rng = np.random.default_rng(w.seed)
    xs32 = (rng.standard_normal((cap, w.H)) * rng.choice([0.05, 1.0, 8.0], (cap, 1))).astype(np.float32)
    xs32[:, 128:256] *= 0.01 if w.H >= 256 else 1.0      # blocks of very different magnitude
    if n > 2:
        xs32[1, :128] = 0.0                                # an all-zero block
    xs = gen.f32_to_bf16_bits(xs32)
    ex = gen.make_local_experts(w)
    ws = torch.empty(moe.moe_fp8act_workspace_bytes(cfg, n_exp, cap), dtype=torch.uint8, device="cuda")
    ys = torch.full((cap, w.H), 7.0, dtype=torch.bfloat16, device="cuda")
    moe.moe_expert_ffn_fp8act(cfg, n_exp, dev(xs), dev(offsets), cap, dev(ex["w_gate"]), dev(ex["w_up"]),
                              dev(ex["w_down"]), dev(ex["s_gate"]), dev(ex["s_up"]), dev(ex["s_down"]),
                              ys, ws)
    torch.cuda.synchronize()
    ref = oracle.expert_ffn_fp8act(offsets, xs, ex["w_gate"], ex["w_up"], ex["w_down"],
                                   ex["s_gate"], ex["s_up"], ex["s_down"])
    got = oracle.decode(host(ys))
    assert np.all(got[n:] == 7.0), "rows past the last valid one were written"
    return got[:n], ref[:n], n, xs, ws, cap


BASE = gen.CONFIGS["c5"].replace(zipf_s=None, shared_expert=False, tp=1, n_groups=1, topk_groups=1,
                                 group_score_n=0)
CASES = {
    # one tile and a ragged tail, several K blocks
    "small": (BASE.replace(name="f8a_small", H=256, I=128, E=4, k=2, expert_lo=0, expert_hi=4, seed=71),
              [5, 0, 130, 1]),
    # several M tiles per expert, N tiles in both GEMMs, an empty expert
    "tiles": (BASE.replace(name="f8a_tiles", H=512, I=384, E=8, k=2, expert_lo=2, expert_hi=6, seed=72),
              [300, 0, 129, 64]),
    # long K (many scale blocks)
    "long_k": (BASE.replace(name="f8a_longk", H=2048, I=256, E=2, k=1, expert_lo=0, expert_hi=2, seed=73),
               [70, 33]),
}


@pytest.mark.parametrize("name", list(CASES))
def test_fp8act_ffn_matches_oracle(name):
    w, counts = CASES[name]
    got, ref, n, _, _, _ = run_case(w, counts)
    err = rel_err(got, ref)
    print(name, "rows", n, "max|err|/max|ref| = %.3e" % err, flush=True)
    assert err <= 6e-2, err
    # typical error is far below the bar: the mean absolute error stays under 1 % of the largest value
    assert np.abs(got - ref).mean() <= 1e-2 * np.abs(ref).max()


def test_fp8act_quantiser_is_bit_exact():
    """The first stage of the call (codes and scales of the input rows, read back
    from the workspace) against the oracle's quantiser: same fp32 decisions."""
    w, counts = CASES["tiles"]
    _, _, n, xs, ws, cap = run_case(w, counts)
    codes_ref, scales_ref = oracle.quant_act_1x128(xs[:n])
    max_tiles = cap // 128 + (w.e_hi - w.expert_lo) + 1
    off = (1 + 4 * max_tiles) * 4
    off = (off + 255) // 256 * 256
    codes = host(ws[off:off + cap * w.H]).reshape(cap, w.H)[:n]
    off2 = off + (cap * w.H + 255) // 256 * 256
    nb = w.H // 128
    scales_t = host(ws[off2:off2 + nb * cap * 4]).view(np.float32).reshape(nb, cap)[:, :n]
    assert np.array_equal(scales_t.T, scales_ref)
    same = (codes == codes_ref) | (((codes | codes_ref) & 0x7F) == 0)      # +0 and -0 are one value
    assert same.all(), "%d codes differ" % (~same).sum()


def test_fp8act_argument_validation():
    w, _ = CASES["small"]
    cfg = config_from_workload(w)
    assert moe.moe_fp8act_workspace_bytes(cfg, 4, 100) > 0
    bad = config_from_workload(w.replace(H=192))
    assert moe.moe_fp8act_workspace_bytes(bad, 4, 100) == 0
    bf = config_from_workload(w.replace(weight_dtype="bf16"))
    assert moe.moe_fp8act_workspace_bytes(bf, 4, 100) == 0


def test_quantise_once_path_equals_the_fused_call():
    """moe_quant_act + moe_dispatch_fp8q + moe_expert_ffn_fp8q against the oracle's
    quantiser and dispatch (bit-exact) and against moe_dispatch + moe_expert_ffn_fp8act
    (the same bits: a row is quantised the same way before or after it is copied)."""
    w = BASE.replace(name="f8a_once", T=333, H=384, I=256, E=12, k=3, expert_lo=2, expert_hi=9, seed=75)
    cfg = config_from_workload(w)
    T, k, H, A, El = w.T, w.k, w.H, w.T * w.k, w.e_hi - w.expert_lo
    rng = np.random.default_rng(9)
    x_np = gen.make_x(w)
    ids = rng.integers(0, w.E, (T, k)).astype(np.int32)
    ex = gen.make_local_experts(w)
    dw = [dev(ex[n]) for n in ("w_gate", "w_up", "w_down", "s_gate", "s_up", "s_down")]
    x = dev(x_np)
    i32 = dict(dtype=torch.int32, device="cuda")
    u8 = dict(dtype=torch.uint8, device="cuda")
    f32 = dict(dtype=torch.float32, device="cuda")
    ws = torch.empty(max(moe.moe_workspace_bytes(cfg, T), moe.moe_fp8act_workspace_bytes(cfg, El, A)), **u8)

    # quantise once
    xq, xq_s = torch.empty(T, H, **u8), torch.empty(H // 128, T, **f32)
    moe.moe_quant_act(cfg, T, x, xq, xq_s)
    torch.cuda.synchronize()
    codes_ref, scales_ref = oracle.quant_act_1x128(x_np)
    got_c = host(xq)
    assert (((got_c == codes_ref) | (((got_c | codes_ref) & 0x7F) == 0))).all()
    assert np.array_equal(host(xq_s).T, scales_ref)

    # dispatch the codes
    counts, offsets = torch.empty(El, **i32), torch.empty(El + 1, **i32)
    perm, inv = torch.empty(A, **i32), torch.empty(A, **i32)
    xs_q, xs_s = torch.zeros(A, H, **u8), torch.zeros(H // 128, A, **f32)
    moe.moe_dispatch_fp8q(cfg, T, xq, xq_s, dev(ids), counts, offsets, perm, inv, xs_q, xs_s, ws)
    torch.cuda.synchronize()
    c_ref, o_ref, p_ref, i_ref, _ = oracle.dispatch(ids, None, w.expert_lo, w.e_hi, want_xs=False)
    n = int(o_ref[-1])
    assert np.array_equal(host(counts), c_ref) and np.array_equal(host(offsets), o_ref)
    assert np.array_equal(host(perm)[:n], p_ref) and np.array_equal(host(inv), i_ref)
    assert np.array_equal(host(xs_q)[:n], got_c[p_ref // k])
    assert np.array_equal(host(xs_s)[:, :n], host(xq_s)[:, p_ref // k])

    # FFN on the dispatched codes == FFN that quantises the dispatched bf16 rows itself
    ys_a = torch.zeros(A, H, dtype=torch.bfloat16, device="cuda")
    moe.moe_expert_ffn_fp8q(cfg, El, xs_q, xs_s, offsets, A, *dw, ys_a, ws)
    xs = torch.zeros(A, H, dtype=torch.bfloat16, device="cuda")
    c2, o2, p2, i2 = (torch.empty_like(t) for t in (counts, offsets, perm, inv))
    moe.moe_dispatch(cfg, T, x, dev(ids), c2, o2, p2, i2, xs, ws)
    ys_b = torch.zeros(A, H, dtype=torch.bfloat16, device="cuda")
    moe.moe_expert_ffn_fp8act(cfg, El, xs, o2, A, *dw, ys_b, ws)
    torch.cuda.synchronize()
    assert torch.equal(ys_a[:n].view(torch.int16), ys_b[:n].view(torch.int16))
    ref = oracle.expert_ffn_fp8act(o_ref, x_np[p_ref // k], ex["w_gate"], ex["w_up"], ex["w_down"],
                                   ex["s_gate"], ex["s_up"], ex["s_down"])
    assert rel_err(oracle.decode(host(ys_a))[:n], ref[:n]) <= 6e-2
