"""Shared plumbing of the GPU parity tests: build inputs once, run the HIP
path through the C ABI, run the oracle, compare."""
import functools

import numpy as np
import torch

import oracle
from workloads import gen

TOL = {"f32": 1e-5, "bf16": 2e-2, "fp8": 6e-2}     # max|err| / max|ref| per weight dtype


@functools.lru_cache(maxsize=2)
def inputs(w):
    """All seeded tensors of a workload (numpy storage form)."""
    d = {"x": gen.make_x(w), "gate": gen.make_gate(w), "experts": gen.make_local_experts(w),
         "shared": gen.make_shared_expert(w) if w.shared_expert else None, "forced": None}
    if w.zipf_s is not None:
        d["forced"] = gen.make_forced_routing(w)
    return d


def oracle_route(w, x, gate, logits_in=None):
    return oracle.route(x, gate["gate_w"], w.k, w.score_fn, w.renormalize, w.routed_scale,
                        w.n_groups, w.topk_groups, w.group_score_n, gate["logit_bias"],
                        gate["select_bias"], logits_in=logits_in)


def make_layer(w, d):
    from paper_2601_08800_amd import MoELayerShare
    from paper_2601_08800_amd.layer import config_from_workload
    cfg = config_from_workload(w)
    return MoELayerShare(cfg, w.T, d["gate"], d["experts"], d["shared"],
                         fp8_activations=w.fp8_activations)


def dev(a):
    from paper_2601_08800_amd.layer import to_device
    return to_device(a)


def host(t):
    """device tensor -> numpy in storage form (bf16 -> uint16 bits)."""
    t = t.detach().cpu()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def check_routing(ids_gpu, w_gpu, ids_ref, w_ref, margin, scale, label=""):
    """ids bit-exact (tokens whose decisive gap is below fp64 resolution may take
    either side and are counted); weights to fp32 accuracy."""
    ambiguous = margin < 1e-9
    bad = np.any(ids_gpu != ids_ref, axis=1) & ~ambiguous
    assert not bad.any(), "%s: %d tokens with wrong ids, first %s" % (
        label, bad.sum(), np.nonzero(bad)[0][:5])
    ok = ~np.any(ids_gpu != ids_ref, axis=1)
    np.testing.assert_allclose(w_gpu[ok], w_ref[ok], rtol=2e-5, atol=2e-6 * scale)
    return int(ambiguous.sum())


def check_dispatch(L, ids, w, x_np, want_rows=True):
    """counts / offsets / perm / inv bit-exact against the oracle; every valid
    row of the send buffer is a bit copy of its token's row (compared on the
    device in chunks, against the input rows gathered through the ORACLE's
    permutation)."""
    c, o, perm, inv, _ = oracle.dispatch(ids, None, w.expert_lo, w.e_hi, want_xs=False)
    n = int(o[-1])
    assert np.array_equal(host(L.counts), c)
    assert np.array_equal(host(L.offsets), o)
    assert np.array_equal(host(L.perm)[:n], perm)
    assert np.array_equal(host(L.inv), inv)
    if want_rows and n:
        k = w.k
        device = L.perm.device
        src = torch.from_numpy(perm // k).to(device)
        if w.fp8_activations:
            # dispatch copied the tokens' e4m3 codes and block scales: every row
            # against the quantised token buffer, and that buffer against the
            # oracle's quantiser on a spread of tokens
            for lo in range(0, n, 1 << 16):
                hi = min(n, lo + (1 << 16))
                assert torch.equal(L.xs_q[lo:hi], L.xq[src[lo:hi]])
                assert torch.equal(L.xs_scales[:, lo:hi], L.xq_scales[:, src[lo:hi]])
            toks = np.unique(np.concatenate([np.arange(min(w.T, 64)), np.arange(max(0, w.T - 64), w.T),
                                             np.random.default_rng(1).integers(0, w.T, 1024)]))
            codes, scales = oracle.quant_act_1x128(x_np[toks])
            sel = torch.from_numpy(toks).to(device)
            got = host(L.xq[sel])
            assert (((got == codes) | (((got | codes) & 0x7F) == 0))).all()      # +0 and -0 are one value
            assert np.array_equal(host(L.xq_scales[:, sel]).T, scales)
        else:
            xd = dev(x_np)
            view = (lambda t: t.view(torch.int16)) if xd.dtype == torch.bfloat16 else (lambda t: t.view(torch.int32))
            for lo in range(0, n, 1 << 16):
                hi = min(n, lo + (1 << 16))
                assert torch.equal(view(L.xs[lo:hi]), view(xd[src[lo:hi]])), "send-buffer rows %d..%d" % (lo, hi)
    return c, o, perm, inv


def border_tokens(w, offsets, perm, at_least, seed=7):
    """Tokens for a sampled output check at sizes where the oracle cannot do every
    row: for every local expert the first and the last row of its segment and the
    rows on either side of every possible M-tile border (tile heights are
    multiples of 32 rows; segments longer than 1024 rows: the borders of the
    balanced 160- and 256-row partitions and every multiple of 256), filled up
    with random tokens to `at_least`."""
    rows = set()
    for e in range(len(offsets) - 1):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        m = hi - lo
        if m == 0:
            continue
        cuts = {0, m}
        if m <= 1024:
            cuts.update(range(32, m, 32))
        else:
            cuts.update(range(256, m, 256))
            for bm in (160, 256):
                nt = -(-m // bm)
                step = -(-(-(-m // nt)) // 32) * 32
                cuts.update(range(step, m, step))
        for c in cuts:
            if c > 0:
                rows.add(lo + c - 1)
            if c < m:
                rows.add(lo + c)
    toks = set((perm[np.array(sorted(rows), np.int64)] // w.k).tolist()) if rows else set()
    rng = np.random.default_rng(seed)
    while len(toks) < min(at_least, w.T):
        toks.update(rng.integers(0, w.T, at_least).tolist())
    return np.array(sorted(toks))


def rel_err(a, ref):
    ref = np.asarray(ref, np.float64)
    return float(np.max(np.abs(np.asarray(a, np.float64) - ref)) / max(np.max(np.abs(ref)), 1e-30))


def oracle_out_for_tokens(w, d, tokens, ids, wts):
    """Oracle output rows for a subset of tokens (rows are independent)."""
    x = d["x"][tokens]
    out, _ = oracle.layer_share(x, ids[tokens], wts[tokens], w.expert_lo, w.e_hi, d["experts"],
                                d["shared"], fp8_activations=w.fp8_activations)
    return out
