"""Pins for the oracle's dispatch, expert MLP, combine and storage decoders."""
import numpy as np
import pytest
import scipy.special
import torch

import oracle
from workloads import gen


def _rand_ids(rng, T, E, k):
    return np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)


# ---------------------------------------------------------------- dispatch
@pytest.mark.parametrize("e_lo,e_hi", [(0, 12), (3, 7), (0, 1), (11, 12)])
def test_dispatch_is_stable_sort_of_local_assignments(e_lo, e_hi):
    rng = np.random.default_rng(e_lo * 13 + e_hi)
    T, E, k, H = 37, 12, 3, 8
    ids = _rand_ids(rng, T, E, k)
    x = rng.standard_normal((T, H)).astype(np.float32)
    counts, offsets, perm, inv, xs = oracle.dispatch(ids, x, e_lo, e_hi)
    flat = ids.ravel()
    local = np.nonzero((flat >= e_lo) & (flat < e_hi))[0]
    # library routine: a stable argsort of the local expert ids
    ref_perm = local[np.argsort(flat[local], kind="stable")]
    assert np.array_equal(perm, ref_perm)
    assert np.array_equal(counts, np.bincount(flat[local] - e_lo, minlength=e_hi - e_lo))
    assert offsets[0] == 0 and np.array_equal(np.diff(offsets), counts)
    assert offsets[-1] == len(local)
    # inverse map and -1 for the rest
    assert np.array_equal(inv[perm], np.arange(len(perm)))
    rest = np.setdiff1d(np.arange(T * k), local)
    assert np.all(inv[rest] == -1)
    # rows are bit copies of the token's row
    assert np.array_equal(xs, x[perm // k])
    # expert of each position matches its segment
    seg = np.repeat(np.arange(e_hi - e_lo), counts) + e_lo
    assert np.array_equal(flat[perm], seg)


def test_dispatch_counts_sum_over_ranges():
    rng = np.random.default_rng(1)
    T, E, k = 50, 16, 4
    ids = _rand_ids(rng, T, E, k)
    x = np.zeros((T, 4), np.float32)
    tot = 0
    for r in range(4):
        c, o, p, inv, xs = oracle.dispatch(ids, x, 4 * r, 4 * r + 4)
        tot += c.sum()
    assert tot == T * k


def test_dispatch_empty():
    ids = np.zeros((0, 2), np.int32)
    x = np.zeros((0, 4), np.float32)
    c, o, p, inv, xs = oracle.dispatch(ids, x, 0, 3)
    assert list(c) == [0, 0, 0] and list(o) == [0, 0, 0, 0] and len(p) == 0


# -------------------------------------------------------------- expert MLP
def _mlp_ref(xs, wg, wu, wd):
    """Dense SwiGLU MLP written with library matmuls in fp64."""
    xs, wg, wu, wd = (a.astype(np.float64) for a in (xs, wg, wu, wd))
    g = xs @ wg.T
    u = xs @ wu.T
    return (g * scipy.special.expit(g) * u) @ wd.T


def test_ffn_single_expert_equals_dense_mlp():
    rng = np.random.default_rng(4)
    R, H, I = 13, 24, 40                                # non-square on purpose
    xs = rng.standard_normal((R, H)).astype(np.float32)
    wg = rng.standard_normal((1, I, H)).astype(np.float32) * 0.3
    wu = rng.standard_normal((1, I, H)).astype(np.float32) * 0.3
    wd = rng.standard_normal((1, H, I)).astype(np.float32) * 0.3
    ys = oracle.expert_ffn(np.array([0, R], np.int32), xs, wg, wu, wd)
    np.testing.assert_allclose(ys, _mlp_ref(xs, wg[0], wu[0], wd[0]), rtol=1e-12, atol=1e-13)


def test_ffn_grouped_uses_each_experts_weights_and_rows():
    rng = np.random.default_rng(5)
    H, I, n = 16, 24, 4
    offsets = np.array([0, 3, 3, 10, 12], np.int32)     # one empty expert
    xs = rng.standard_normal((14, H)).astype(np.float32)  # 2 rows of padding
    wg = rng.standard_normal((n, I, H)).astype(np.float32) * 0.3
    wu = rng.standard_normal((n, I, H)).astype(np.float32) * 0.3
    wd = rng.standard_normal((n, H, I)).astype(np.float32) * 0.3
    ys = oracle.expert_ffn(offsets, xs, wg, wu, wd)
    for e in range(n):
        r = slice(offsets[e], offsets[e + 1])
        np.testing.assert_allclose(ys[r], _mlp_ref(xs[r], wg[e], wu[e], wd[e]), rtol=1e-12, atol=1e-13)
    assert np.all(ys[12:] == 0)


def test_ffn_closed_forms():
    rng = np.random.default_rng(6)
    R, H, I = 5, 8, 16
    xs = rng.standard_normal((R, H)).astype(np.float32)
    wg = rng.standard_normal((1, I, H)).astype(np.float32)
    wu = rng.standard_normal((1, I, H)).astype(np.float32)
    wd = rng.standard_normal((1, H, I)).astype(np.float32)
    off = np.array([0, R], np.int32)
    assert np.all(oracle.expert_ffn(off, xs, wg, 0 * wu, wd) == 0)      # Wup = 0
    assert np.all(oracle.expert_ffn(off, xs, 0 * wg, wu, wd) == 0)      # silu(0) = 0
    a = oracle.expert_ffn(off, xs, wg, wu, wd)
    b = oracle.expert_ffn(off, xs, wg, wu, 2 * wd)                      # linear in Wdown
    np.testing.assert_allclose(b, 2 * a, rtol=1e-14)
    # large positive gate: silu(g) -> g, so ys -> Wdown ((Wgate x) * (Wup x))
    xs1 = np.ones((1, H), np.float32)
    wg1 = np.full((1, I, H), 10.0, np.float32)
    ys = oracle.expert_ffn(np.array([0, 1], np.int32), xs1, wg1, wu, wd)
    g = 10.0 * H
    ref = wd[0].astype(np.float64) @ (g * (wu[0].astype(np.float64) @ np.ones(H)))
    np.testing.assert_allclose(ys[0], ref, rtol=1e-12)


def test_ffn_tp_additivity():
    # slicing I into contiguous blocks and summing the partial outputs gives
    # the un-sliced result (block matrix multiplication)
    rng = np.random.default_rng(7)
    R, H, I = 6, 12, 32
    xs = rng.standard_normal((R, H)).astype(np.float32)
    wg = rng.standard_normal((2, I, H)).astype(np.float32) * 0.3
    wu = rng.standard_normal((2, I, H)).astype(np.float32) * 0.3
    wd = rng.standard_normal((2, H, I)).astype(np.float32) * 0.3
    off = np.array([0, 2, R], np.int32)
    full = oracle.expert_ffn(off, xs, wg, wu, wd)
    acc = 0
    for r in range(4):
        s = slice(r * 8, (r + 1) * 8)
        acc = acc + oracle.expert_ffn(off, xs, wg[:, s].copy(), wu[:, s].copy(), wd[:, :, s].copy())
    np.testing.assert_allclose(acc, full, rtol=1e-12, atol=1e-14)


def test_ffn_block_scales():
    # a 3 x 2 grid of blocks (I = 384, H = 256) with a different power of two in every
    # block, so that a transposed or shifted block index changes the result
    rng = np.random.default_rng(8)
    R, H, I = 3, 256, 384
    xs = rng.standard_normal((R, H)).astype(np.float32)
    wg = rng.standard_normal((1, I, H)).astype(np.float32)
    wu = rng.standard_normal((1, I, H)).astype(np.float32)
    wd = rng.standard_normal((1, H, I)).astype(np.float32)
    sg = np.array([[[0.5, 2.0], [8.0, 0.125], [1.0, 32.0]]], np.float32)       # [1, I/128, H/128]
    su = np.array([[[4.0, 0.25], [0.5, 16.0], [2.0, 0.0625]]], np.float32)
    sd = np.array([[[2.0, 0.5, 64.0], [8.0, 0.25, 1.0]]], np.float32)          # [1, H/128, I/128]
    ys = oracle.expert_ffn(np.array([0, R], np.int32), xs, wg, wu, wd, sg, su, sd)
    blow = lambda s: np.kron(s[0], np.ones((128, 128), np.float32))            # power-of-two scales: exact
    ref = _mlp_ref(xs, wg[0] * blow(sg), wu[0] * blow(su), wd[0] * blow(sd))
    np.testing.assert_allclose(ys, ref, rtol=1e-11, atol=1e-12 * np.abs(ref).max())


# ----------------------------------------------------------------- combine
def test_combine_weighted_gather():
    rng = np.random.default_rng(9)
    T, k, H = 7, 3, 5
    inv = rng.permutation(T * k).astype(np.int32)
    inv[[2, 5, 11]] = -1
    ys = rng.standard_normal((T * k, H))
    w = rng.random((T, k)).astype(np.float32)
    sh = rng.standard_normal((T, H))
    out = oracle.combine(ys, inv, w, sh)
    iv = inv.reshape(T, k)
    ref = np.zeros((T, H))
    for t in range(T):
        for j in range(k):
            if iv[t, j] >= 0:
                ref[t] += np.float64(w[t, j]) * ys[iv[t, j]]
    ref += sh
    np.testing.assert_allclose(out, ref.astype(np.float32), rtol=1e-6)
    # linear in w; shared only when every assignment is remote
    out2 = oracle.combine(ys, inv, 2 * w, None)
    np.testing.assert_allclose(out2, 2 * oracle.combine(ys, inv, w, None), rtol=1e-6)
    out3 = oracle.combine(ys, np.full(T * k, -1, np.int32), w, sh)
    assert np.array_equal(out3, sh.astype(np.float32))
    # a rank that received no row at all (an empty buffer of the right width): the
    # sum over no experts is zero, with the layer's full shape
    none = oracle.combine(np.zeros((0, H)), np.full(T * k, -1, np.int32), w, None)
    assert none.shape == (T, H) and not none.any()


def test_layer_share_with_no_local_assignment():
    rng = np.random.default_rng(21)
    T, H, E, k, I = 9, 16, 12, 3, 8
    x = rng.standard_normal((T, H)).astype(np.float32)
    ids = rng.integers(0, 5, (T, k)).astype(np.int32)          # nothing goes to experts 7..8
    w = rng.random((T, k)).astype(np.float32)
    ex = {"w_gate": rng.standard_normal((2, I, H)).astype(np.float32),
          "w_up": rng.standard_normal((2, I, H)).astype(np.float32),
          "w_down": rng.standard_normal((2, H, I)).astype(np.float32)}
    out, parts = oracle.layer_share(x, ids, w, 7, 9, ex)
    assert out.shape == (T, H) and not out.any()
    assert parts["counts"].tolist() == [0, 0] and (parts["inv"] == -1).all()


def test_identity_experts_return_input():
    # bypassing the MLP (ys := xs) the layer returns (sum of weights) * x
    rng = np.random.default_rng(10)
    T, H, E, k = 33, 16, 8, 2
    x = rng.standard_normal((T, H)).astype(np.float32)
    gw = rng.standard_normal((E, H)).astype(np.float32)
    ids, w, _ = oracle.route(x, gw, k)
    c, o, perm, inv, xs = oracle.dispatch(ids, x, 0, E)
    assert c.sum() == T * k
    out = oracle.combine(xs.astype(np.float64), inv, w)
    np.testing.assert_allclose(out, x, rtol=1e-6, atol=1e-7)
    ids, w, _ = oracle.route(x, gw, k, "sigmoid", routed_scale=2.5)
    c, o, perm, inv, xs = oracle.dispatch(ids, x, 0, E)
    out = oracle.combine(xs.astype(np.float64), inv, w)
    np.testing.assert_allclose(out, 2.5 * x, rtol=1e-6, atol=1e-7)


def test_ep_additivity_of_layer_share():
    # experts are independent MLPs: the partial outputs of the EP ranges add
    # up to the full layer
    rng = np.random.default_rng(12)
    T, H, E, k, I = 20, 16, 8, 3, 24
    x = rng.standard_normal((T, H)).astype(np.float32)
    gw = rng.standard_normal((E, H)).astype(np.float32)
    W = {"w_gate": rng.standard_normal((E, I, H)).astype(np.float32) * 0.3,
         "w_up": rng.standard_normal((E, I, H)).astype(np.float32) * 0.3,
         "w_down": rng.standard_normal((E, H, I)).astype(np.float32) * 0.3}
    ids, w, _ = oracle.route(x, gw, k)
    full, _ = oracle.layer_share(x, ids, w, 0, E, W)
    acc = np.zeros((T, H))
    for r in range(4):
        sub = {n: a[2 * r:2 * r + 2].copy() for n, a in W.items()}
        part, _ = oracle.layer_share(x, ids, w, 2 * r, 2 * r + 2, sub)
        acc += part
    np.testing.assert_allclose(acc, full, rtol=2e-6, atol=1e-7)
    # dense reference: out[t] = sum_j w[t,j] * MLP_{ids[t,j]}(x[t])
    ref = np.zeros((T, H))
    for t in range(T):
        for j in range(k):
            e = ids[t, j]
            ref[t] += np.float64(w[t, j]) * _mlp_ref(x[t:t + 1], W["w_gate"][e], W["w_up"][e], W["w_down"][e])[0]
    np.testing.assert_allclose(full, ref, rtol=2e-6, atol=1e-7)


# ---------------------------------------------------------------- decoders
def test_e4m3_decode_matches_library_and_roundtrip():
    codes = np.arange(256, dtype=np.uint8)
    dec = oracle.decode(codes)
    lib = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).to(torch.float32).numpy()
    finite = ~np.isnan(lib)
    assert finite.sum() == 254 and np.isnan(dec[~finite]).all()
    assert np.array_equal(dec[finite], lib[finite])
    assert dec[0x7E] == 448.0 and dec[0x01] == 2.0 ** -9 and dec[0x08] == 2.0 ** -6
    # the generator's encoder inverts the decoder on every finite code
    enc = gen.f32_to_e4m3_codes(dec[finite])
    ok = codes[finite]
    same = (enc == ok) | ((dec[finite] == 0) & ((enc & 0x7F) == 0))
    assert same.all()


def test_e4m3_encoder_matches_library_rounding():
    rng = np.random.default_rng(13)
    v = np.concatenate([rng.standard_normal(20000) * 100, rng.standard_normal(20000) * 0.02,
                        [448.0, 464.0, 500.0, -1e4, 0.0, 2.0 ** -10, 3 * 2.0 ** -10]]).astype(np.float32)
    v = np.clip(v, -448, 448)
    lib = torch.from_numpy(v).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    enc = gen.f32_to_e4m3_codes(v)
    dz = oracle.decode(enc)
    assert np.array_equal(dz, oracle.decode(lib))


def test_bf16_codec_matches_library():
    rng = np.random.default_rng(14)
    v = (rng.standard_normal(50000) * np.exp(rng.uniform(-20, 20, 50000))).astype(np.float32)
    bits = gen.f32_to_bf16_bits(v)
    lib = torch.from_numpy(v).to(torch.bfloat16)
    assert np.array_equal(bits, lib.view(torch.int16).numpy().view(np.uint16))
    assert np.array_equal(oracle.decode(bits), lib.to(torch.float32).numpy())


def test_fp8_block_quantiser():
    rng = np.random.default_rng(15)
    w = (rng.standard_normal((256, 384)) * 0.02).astype(np.float32)
    codes, scales = gen.quantize_e4m3_block128(w)
    assert scales.shape == (2, 3)
    deq = oracle.decode(codes).astype(np.float64) * np.repeat(np.repeat(scales, 128, 0), 128, 1)
    assert np.max(np.abs(deq - w)) <= np.max(np.abs(w)) / 16 + 1e-9   # half a 3-bit-mantissa step
    assert np.abs(oracle.decode(codes)).max() == 448.0
    # exactly representable weights with unit scale survive unchanged
    grid = oracle.decode(np.arange(0, 0x7F, dtype=np.uint8))
    w2 = np.tile(grid, (128, 2))[:, :128].copy()
    w2[0, 0] = 448.0
    c2, s2 = gen.quantize_e4m3_block128(w2)
    assert s2[0, 0] == 1.0 and np.array_equal(oracle.decode(c2), w2)


def test_frozen_tiny_layer_and_hand_check():
    """The stored fixture (written by tests/golden/make_golden.py from the oracle
    alone) still matches, and its first token is re-derived by hand here."""
    import os
    import sys
    gdir = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    sys.path.insert(0, gdir)
    import make_golden
    ids, w, offsets, perm, out = make_golden.compute()
    rec = {}
    for line in open(os.path.join(gdir, "tiny_layer.txt")):
        if not line.startswith("#"):
            key, *vals = line.split()
            rec[key] = vals
    assert list(map(int, rec["ids"])) == list(ids.ravel())
    assert list(map(int, rec["offsets"])) == list(offsets)
    assert list(map(int, rec["perm"])) == list(perm)
    np.testing.assert_allclose(np.array(rec["w"], np.float64), w.ravel(), rtol=1e-7)
    np.testing.assert_allclose(np.array(rec["out"], np.float64), out.ravel(), rtol=1e-6, atol=1e-9)
    # token 0 by hand: logits, top-2, softmax over the two, two tiny MLPs
    x, gw, W, k = make_golden.tiny_inputs()
    z = [float(np.dot(x[0].astype(np.float64), gw[e].astype(np.float64))) for e in range(4)]
    top = sorted(range(4), key=lambda e: (-z[e], e))[:2]
    assert top == list(ids[0])
    p = np.exp(np.array([z[e] for e in top]) - max(z))
    p /= p.sum()
    acc = np.zeros(4)
    for e, pw in zip(top, p):
        g = W["w_gate"][e].astype(np.float64) @ x[0]
        u = W["w_up"][e].astype(np.float64) @ x[0]
        acc += np.float32(pw).astype(np.float64) * (W["w_down"][e].astype(np.float64) @ (g / (1 + np.exp(-g)) * u))
    np.testing.assert_allclose(out[0], acc, rtol=1e-6, atol=1e-9)
