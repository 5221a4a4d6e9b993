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
    """counts / offsets / perm / inv bit-exact against the oracle; xs rows are
    bit copies."""
    c, o, perm, inv, _ = oracle.dispatch(ids, None, w.expert_lo, w.e_hi, want_xs=False)
    n = int(o[-1])
    assert np.array_equal(host(L.counts), c)
    assert np.array_equal(host(L.offsets), o)
    assert np.array_equal(host(L.perm)[:n], perm)
    assert np.array_equal(host(L.inv), inv)
    if want_rows and n:
        k = w.k
        rows = np.unique(np.concatenate([np.arange(min(n, 64)), np.arange(max(0, n - 64), n),
                                         np.random.default_rng(1).integers(0, n, 256)]))
        sel = torch.from_numpy(rows).to(L.xs.device)
        if w.fp8_activations:      # dispatch copied the tokens' e4m3 codes and block scales
            codes, scales = oracle.quant_act_1x128(x_np[perm[rows] // k])
            got = host(L.xs_q[sel])
            assert (((got == codes) | (((got | codes) & 0x7F) == 0))).all()
            assert np.array_equal(host(L.xs_scales[:, sel]).T, scales)
        else:
            assert np.array_equal(host(L.xs[sel]), x_np[perm[rows] // k])
    return c, o, perm, inv


def rel_err(a, ref):
    ref = np.asarray(ref, np.float64)
    return float(np.max(np.abs(np.asarray(a, np.float64) - ref)) / max(np.max(np.abs(ref)), 1e-30))


def oracle_out_for_tokens(w, d, tokens, ids, wts):
    """Oracle output rows for a subset of tokens (rows are independent)."""
    x = d["x"][tokens]
    out, _ = oracle.layer_share(x, ids[tokens], wts[tokens], w.expert_lo, w.e_hi, d["experts"],
                                d["shared"], fp8_activations=w.fp8_activations)
    return out
