"""Pins of the oracle's 8-bit-activation functions (CPU): the quantiser against
the library's e4m3 rounding and the properties its definition fixes, the FFN
against a composition of library routines (library e4m3 rounding, numpy fp64
products; the intermediate goes to the quantiser unrounded) and against the
unquantised FFN."""
import numpy as np
import torch

import oracle
from workloads import gen


def lib_e4m3(q):
    return torch.from_numpy(np.ascontiguousarray(q, np.float32)).to(torch.float8_e4m3fn)


def test_quantiser_matches_library_rounding_and_its_definition():
    rng = np.random.default_rng(5)
    x = (rng.standard_normal((64, 384)) * rng.choice([1e-3, 1.0, 50.0], (64, 1))).astype(np.float32)
    x[3, 128:256] = 0.0                                  # all-zero block
    x[4, :128] = 2.0 ** -20                              # constant block
    x[5, 7] = 1000.0                                     # an outlier sets its block's scale
    codes, scales = oracle.quant_act_1x128(x)
    xb = x.reshape(64, 3, 128)
    amax = np.abs(xb).max(axis=2)
    want_scale = np.where(amax > 0, amax / np.float32(448.0), np.float32(1.0)).astype(np.float32)
    assert np.array_equal(scales, want_scale)
    q = np.clip(xb / scales[:, :, None], -448, 448).astype(np.float32)
    lib = lib_e4m3(q).view(torch.uint8).numpy().reshape(64, 384)
    assert np.array_equal(codes, lib)
    # the block's largest element becomes +-448
    dec = oracle.decode(codes).reshape(64, 3, 128)
    assert np.all(np.abs(dec).max(axis=2)[amax > 0] == 448.0)
    assert not codes[3, 128:256].any() and scales[3, 1] == 1.0
    # round trip: half a step of a 3-bit mantissa, or half a subnormal step
    back = dec.astype(np.float64) * scales[:, :, None]
    err = np.abs(back - xb)
    assert np.all(err <= np.maximum(np.abs(xb) * 2.0 ** -4, scales[:, :, None] * 2.0 ** -10) * (1 + 1e-6))
    # values on the e4m3 grid with a power-of-two amax / 448 survive exactly
    grid = oracle.decode(np.arange(0, 0x7F, dtype=np.uint8))
    row = np.zeros((1, 128), np.float32)
    row[0, :127] = grid * 4.0
    row[0, 127] = -448.0 * 4.0
    c2, s2 = oracle.quant_act_1x128(row)
    assert s2[0, 0] == 4.0 and np.array_equal(oracle.decode(c2)[0] * 4.0, row[0])


def _case(seed, n=2, H=256, I=128, rows=(9, 5)):
    w = gen.CONFIGS["c5"].replace(name="pin", H=H, I=I, E=n, k=1, expert_lo=0, expert_hi=n, tp=1,
                                  shared_expert=False, zipf_s=None, seed=seed)
    ex = gen.make_local_experts(w)
    rng = np.random.default_rng(seed)
    offsets = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    xs = gen.f32_to_bf16_bits(rng.standard_normal((int(offsets[-1]), H)).astype(np.float32))
    return w, ex, offsets, xs


def _weights(ex, name, sname, e):
    wq = oracle.decode(ex[name][e]).astype(np.float64)
    s = ex[sname][e].astype(np.float64)
    return wq * np.kron(s, np.ones((128, 128)))[:wq.shape[0], :wq.shape[1]]


def test_ffn_equals_a_composition_of_library_routines():
    # 3 x 2 blocks of weight scales, two blocks of hidden-activation scales
    w, ex, offsets, xs = _case(31, H=384, I=256)
    ys = oracle.expert_ffn_fp8act(offsets, xs, ex["w_gate"], ex["w_up"], ex["w_down"],
                                  ex["s_gate"], ex["s_up"], ex["s_down"])

    def quant(a32):                                     # library rounding, numpy scales
        r, K = a32.shape
        b = a32.reshape(r, K // 128, 128)
        amax = np.abs(b).max(axis=2, keepdims=True)
        s = np.where(amax > 0, amax / np.float32(448.0), np.float32(1.0)).astype(np.float32)
        q = np.clip(b / s, -448, 448).astype(np.float32)
        return (lib_e4m3(q).to(torch.float32).numpy().astype(np.float64) * s).reshape(r, K)

    x32 = oracle.decode(xs)
    for e in range(2):
        lo, hi = offsets[e], offsets[e + 1]
        xq = quant(x32[lo:hi])
        g = xq @ _weights(ex, "w_gate", "s_gate", e).T
        u = xq @ _weights(ex, "w_up", "s_up", e).T
        hm = g / (1 + np.exp(-g)) * u
        ref = quant(hm.astype(np.float32)) @ _weights(ex, "w_down", "s_down", e).T
        np.testing.assert_allclose(ys[lo:hi], ref, rtol=1e-9, atol=1e-12 * np.abs(ref).max())


def test_ffn_stays_close_to_the_unquantised_ffn_and_closed_forms():
    w, ex, offsets, xs = _case(32, rows=(40, 24))
    args = (ex["w_gate"], ex["w_up"], ex["w_down"], ex["s_gate"], ex["s_up"], ex["s_down"])
    ys = oracle.expert_ffn_fp8act(offsets, xs, *args)
    plain = oracle.expert_ffn(offsets, xs, *args)
    # 3-bit mantissas on both activations: a few per cent of the largest value at most
    assert np.abs(ys - plain).max() <= 5e-2 * np.abs(plain).max()
    assert np.abs(ys - plain).mean() <= 1e-2 * np.abs(plain).max()
    # an all-zero up projection gives zero, whatever the quantisation does
    zero_up = np.zeros_like(ex["w_up"])
    assert not oracle.expert_ffn_fp8act(offsets, xs, ex["w_gate"], zero_up, ex["w_down"],
                                        ex["s_gate"], ex["s_up"], ex["s_down"]).any()
    # rows are independent: a row computed alone equals the row in the batch
    one = oracle.expert_ffn_fp8act(np.array([0, 1, 1], np.int32), xs[3:4], *args)
    assert np.array_equal(one[0], ys[3])
    # scaling a row by a power of two scales its output (scales absorb it exactly)... for the
    # linear part only; the gate is not linear, so check the quantiser alone
    c1, s1 = oracle.quant_act_1x128(oracle.decode(xs)[:4])
    c2, s2 = oracle.quant_act_1x128(oracle.decode(xs)[:4] * 8.0)
    assert np.array_equal(c1, c2) and np.array_equal(s2, s1 * 8.0)
