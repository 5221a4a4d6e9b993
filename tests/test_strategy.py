"""The analytic strategy selector (host code, no GPU): the Python reference is
pinned to what the paper's text and textbook queueing theory fix, and the C
implementation is compared with it field by field."""
import ctypes
import math
import os
import re

import numpy as np
import pytest

import paper_2601_08800_amd as moe
from paper_2601_08800_amd import strategy as S
from oracle import strategy_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GB = 1e9


def cluster(**kw):
    d = dict(n_node=4, n_proc=8, mem_bytes=288 * GB, bw_intra=400 * GB, bw_inter=50 * GB,
             bw_p2p=50 * GB, compute_rate=1e18)
    d.update(kw)
    return d


def model(**kw):
    d = dict(psi_attn=22 * GB, psi_moe=1300 * GB, layers=61, hidden=7168, top_k=8, act_bytes=2.0)
    d.update(kw)
    return d


def mix(**kw):
    d = dict(batch=16, len_in=4096, len_out=256, arrival_rate=0.0, max_ttft=0.0, max_itl=0.0)
    d.update(kw)
    return d


def c_args(cl, mo, rq):
    return S.MoECluster(**cl), S.MoEModel(**mo), S.MoERequestMix(**rq)


# ---------------------------------------------------------------- ABI
def test_header_symbols_are_exported():
    hdr = open(os.path.join(ROOT, "include", "moe_strategy.h")).read()
    declared = set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", hdr))
    assert declared == set(S.STRATEGY_EXPORTS)
    lib = ctypes.CDLL(moe.lib_path())
    for name in declared:
        assert getattr(lib, name) is not None


@pytest.mark.parametrize("cls,name", [(S.MoECluster, "moe_cluster"), (S.MoEModel, "moe_model"),
                                      (S.MoERequestMix, "moe_request_mix"),
                                      (S.MoEStrategy, "moe_strategy")])
def test_struct_mirrors_match_header(cls, name):
    hdr = open(os.path.join(ROOT, "include", "moe_strategy.h")).read()
    end = hdr.index("} %s;" % name)
    body = hdr[hdr.rindex("typedef struct {", 0, end):end]
    fields = []
    for typ, names in re.findall(r"^\s*(int32_t|double)\s+([\w, ]+);", body, re.M):
        fields += [(n.strip(), typ) for n in names.split(",")]
    assert [f[0] for f in fields] == [f[0] for f in cls._fields_]
    for (n, typ), (_, ct) in zip(fields, cls._fields_):
        assert ct is (ctypes.c_int32 if typ == "int32_t" else ctypes.c_double), n


# ------------------------------------------------------ pins of the reference
def test_pairwise_all_to_all_is_d_minus_one_rounds():
    # Sec. III-A-2: the pairwise algorithm takes d-1 rounds, each moving the block
    # meant for one peer (size / d): play the rounds out
    for d in (1, 2, 4, 8, 32):
        size, bw = 3.0e9, 5.0e10
        t = 0.0
        for rnd in range(1, d):
            sent = [size / d for rank in range(d)]         # rank -> (rank + rnd) % d
            t += max(sent) / bw
        assert math.isclose(O.A2A(size, d, bw), t, rel_tol=1e-12, abs_tol=0.0)
    assert O.A2A(123.0, 1, 1.0) == 0.0


def test_one_round_scatter_and_gather():
    # "Broadcast" RS / AG: every device exchanges a 1/d slice with every peer over
    # its own full-duplex link, all at once: one round of size / d
    size, bw = 8.0e8, 1.0e11
    for d in (2, 4, 8):
        per_link = [size / d for peer in range(d - 1)]
        assert math.isclose(O.RS(size, d, bw), max(per_link) / bw, rel_tol=1e-12)
        assert O.AG(size, d, bw) == O.RS(size, d, bw)
    assert O.RS(size, 1, bw) == 0.0
    # AR as printed: RS and AG of size / d  ->  2 size / d^2
    assert math.isclose(O.AR(size, 4, bw), 2 * size / 16 / bw, rel_tol=1e-12)


def test_queue_is_textbook_mm1():
    cl, mo = cluster(), model()
    base = O.evaluate(cl, mo, mix(), 8, 4, 4, 1)
    mu = 1.0 / base["svc_dec"]
    for rho in (0.1, 0.5, 0.9):
        s = O.evaluate(cl, mo, mix(arrival_rate=rho * mu), 8, 4, 4, 1)
        # mean number waiting L_q = rho^2 / (1 - rho), and Little's law L_q = lambda_a W_q
        assert math.isclose(s["wq"] * rho * mu, rho * rho / (1 - rho), rel_tol=1e-9)
        assert math.isclose(s["ttft"], s["wq"] + s["svc_prf"], rel_tol=1e-12)
    assert O.evaluate(cl, mo, mix(arrival_rate=mu), 8, 4, 4, 1)["wq"] == math.inf
    assert O.evaluate(cl, mo, mix(arrival_rate=2 * mu), 8, 4, 4, 1)["feasible"] == 0
    # mu = 2, lambda_a = 1: W_q = 1 / 2
    assert math.isclose(1.0 / (2.0 * (2.0 - 1.0)), 0.5)


def test_scaling_laws_of_the_latency_terms():
    cl, mo, rq = cluster(), model(), mix()
    a = O.evaluate(cl, mo, rq, 4, 8, 2, 1)
    b = O.evaluate(cl, mo, rq, 4, 8, 4, 1)
    # tau ~ 1 / d_DP, and linear in s
    assert math.isclose(a["tau_prf"], 2 * b["tau_prf"], rel_tol=1e-12)
    assert math.isclose(a["tau_prf"], rq["len_in"] * a["tau_dec"], rel_tol=1e-12)
    assert math.isclose(a["lambda_prf"], rq["len_in"] * a["lambda_dec"], rel_tol=1e-12)
    # the two branches of the A2A term agree where they meet (d_DP = d_EP)
    h, k, eb = mo["hidden"], mo["top_k"], mo["act_bytes"]
    d = 8
    left = O.A2A(rq["batch"] / d * h * k * eb, d, 1.0)
    right = O.A2A(rq["batch"] / d * h * k * eb, d, 1.0)
    assert left == right
    # d_DP < d_EP: groups of d_DP devices exchanging b / d_EP sequences
    s = O.evaluate(cl, mo, rq, 4, 8, 2, 1)
    ar = 2 * (rq["batch"] / 2 * h * eb) / 16 / cl["bw_intra"]
    a2a = (rq["batch"] / 8 * h * k * eb) / 2 * 1 / cl["bw_intra"]     # 4 * 2 = 8 devices: one node
    assert math.isclose(s["lambda_dec"], 2 * ar + 2 * a2a, rel_tol=1e-12)
    # indicators
    assert s["itl"] == s["svc_dec"]
    assert math.isclose(s["throughput"] * (s["wq"] + s["svc_prf"] + rq["len_out"] * s["svc_dec"]),
                        rq["len_in"] + rq["len_out"], rel_tol=1e-12)


def test_compute_term_by_hand():
    # one layer holds (3 + 5) / 4 = 2 bytes of weights; TP 2 x EP 4 leaves 1/4 of them per
    # device; 8 / 2 = 4 sequences of 5 tokens, hidden 10: 1/4 * 4 * 5 * 10 = 50, at rate 2: 25
    cl = cluster(n_node=2, n_proc=4, compute_rate=2.0)
    mo = model(psi_attn=3.0, psi_moe=5.0, layers=4, hidden=10)
    s = O.evaluate(cl, mo, mix(batch=8, len_in=5, len_out=0), 2, 4, 2, 1)
    assert math.isclose(s["tau_prf"], 25.0, rel_tol=1e-12)
    assert math.isclose(s["tau_dec"], 5.0, rel_tol=1e-12)
    # service latency: l layers; three pipeline hops of b/d_DP * s * h * bytes each
    s3 = O.evaluate(cl, mo, mix(batch=8, len_in=5, len_out=0), 2, 4, 2, 4)
    hop = 4 * 5 * 10 * mo["act_bytes"] / cl["bw_p2p"]
    assert math.isclose(s3["svc_prf"], 4 * (s3["tau_prf"] + s3["lambda_prf"]) + 3 * hop, rel_tol=1e-12)
    assert math.isclose(s["svc_prf"], 4 * (s["tau_prf"] + s["lambda_prf"]), rel_tol=1e-12)


def test_memory_constraint_by_hand():
    # 8 GB attention + 64 GB experts, TP 4 x EP 8, no K/V: 2 GB + 2 GB
    cl = cluster(mem_bytes=4.5 * GB)
    mo = model(psi_attn=8 * GB, psi_moe=64 * GB, layers=2, hidden=64, act_bytes=2.0)
    rq = mix(batch=4, len_in=6, len_out=2)
    s = O.evaluate(cl, mo, rq, 4, 8, 4, 1)
    kv = 2 * 4 * 8 * 64 * 2.0 * 2
    assert math.isclose(s["mem_bytes"], 4 * GB + kv, rel_tol=1e-12) and s["feasible"] == 1
    assert O.evaluate(cluster(mem_bytes=4 * GB), mo, rq, 4, 8, 4, 1)["feasible"] == 0
    # two pipeline stages halve the K/V term
    s2 = O.evaluate(cl, mo, rq, 4, 8, 4, 2)
    assert math.isclose(s2["mem_bytes"], 4 * GB + kv / 2, rel_tol=1e-12)


def test_enumeration_on_the_papers_example_cluster():
    # Fig. "An example of TP-EP hybrid parallelism": 2 nodes of 4 devices
    cl = cluster(n_node=2, n_proc=4)
    all_ = O.enumerate_strategies(cl, model(), mix(), 1)
    assert sorted({(s["d_tp"], s["d_ep"]) for s in all_}) == [(1, 8), (2, 4), (4, 2), (8, 1)]
    assert all(s["d_tp"] * s["d_ep"] == 8 and s["d_dp"] * s["d_tp"] <= 8 for s in all_)
    assert len(all_) == 4 + 3 + 2 + 1
    # a batch of 2 cannot be split four ways
    assert max(s["d_dp"] for s in O.enumerate_strategies(cl, model(), mix(batch=2), 1)) == 2


def test_select_is_the_argmax_of_the_enumeration():
    cl, mo, rq = cluster(), model(), mix()
    best = O.select(cl, mo, rq, 1)
    feas = [s for s in O.enumerate_strategies(cl, mo, rq, 1) if s["feasible"]]
    assert best is not None and best["throughput"] == max(s["throughput"] for s in feas)
    assert min(s["d_tp"] for s in feas) == 1
    # K/V cache 121.8 GB + experts 1300/32 GB leave room for the attention weights
    # (22 GB / d_TP) on a 170 GB device only from d_TP = 4 on
    tight = cluster(mem_bytes=170 * GB)
    feas_t = [s for s in O.enumerate_strategies(tight, mo, rq, 1) if s["feasible"]]
    assert feas_t and all(s["d_tp"] >= 4 for s in feas_t)
    assert O.select(tight, mo, rq, 1)["d_tp"] >= 4
    assert O.select(cluster(mem_bytes=1 * GB), mo, rq, 1) is None


def test_hybrid_scheme_moves_less_across_nodes():
    # Sec. III-B-2: lambda_EP - lambda_mix = 2 A2A(bshk, n) (1 - 1/p) - AG(bshk/p, p)
    cl, mo = cluster(n_node=4, n_proc=8), model()
    tokens = 16 * 4096
    bshk = tokens * mo["hidden"] * mo["act_bytes"] * mo["top_k"]
    p, n = cl["n_proc"], cl["n_node"]
    diff = 2 * (bshk / n * (n - 1) / cl["bw_inter"]) * (1 - 1 / p) - bshk / p / p / cl["bw_intra"]
    assert math.isclose(O.lambda_ep(cl, mo, tokens) - O.lambda_mix(cl, mo, tokens), diff, rel_tol=1e-9)
    assert O.lambda_mix(cl, mo, tokens) < O.lambda_ep(cl, mo, tokens)


# ------------------------------------------------ C implementation vs reference
FIELDS = [f for f, _ in S.MoEStrategy._fields_]


def same(c_s, o_s):
    for f in FIELDS:
        a, b = getattr(c_s, f), o_s[f]
        if isinstance(b, float) and math.isinf(b):
            assert math.isinf(a), f
        else:
            assert math.isclose(a, b, rel_tol=1e-12, abs_tol=0.0), (f, a, b)


def random_case(seed):
    r = np.random.default_rng(seed)
    cl = cluster(n_node=int(2 ** r.integers(0, 5)), n_proc=int(2 ** r.integers(0, 4)),
                 mem_bytes=float(r.uniform(20, 400)) * GB, bw_intra=float(r.uniform(100, 900)) * GB,
                 bw_inter=float(r.uniform(10, 100)) * GB, bw_p2p=float(r.uniform(10, 100)) * GB,
                 compute_rate=float(10 ** r.uniform(16, 19)))
    mo = model(psi_attn=float(r.uniform(1, 50)) * GB, psi_moe=float(r.uniform(10, 1500)) * GB,
               layers=int(r.integers(1, 100)), hidden=int(r.integers(1, 64)) * 128,
               top_k=int(r.integers(1, 9)), act_bytes=float(r.choice([1.0, 2.0, 4.0])))
    rq = mix(batch=int(r.integers(1, 300)), len_in=int(r.integers(1, 8000)),
             len_out=int(r.integers(0, 2000)), arrival_rate=float(r.choice([0.0, r.uniform(0, 50)])),
             max_ttft=float(r.choice([0.0, r.uniform(0.01, 10)])),
             max_itl=float(r.choice([0.0, r.uniform(0.001, 1)])))
    return cl, mo, rq, int(r.integers(1, 5))


@pytest.mark.parametrize("seed", range(40))
def test_c_matches_reference_on_random_cases(seed):
    cl, mo, rq, d_pp = random_case(seed)
    ca = c_args(cl, mo, rq)
    ref_all = O.enumerate_strategies(cl, mo, rq, d_pp)
    best, all_ = S.moe_strategy_select(*ca, d_pp=d_pp)
    assert len(all_) == len(ref_all)
    for c_s, o_s in zip(all_, ref_all):
        same(c_s, o_s)
        same(S.moe_strategy_eval(*ca, o_s["d_tp"], o_s["d_ep"], o_s["d_dp"], d_pp), o_s)
    ref_best = O.select(cl, mo, rq, d_pp)
    if ref_best is None:
        assert best is None
    else:
        same(best, ref_best)
    tokens = float(rq["batch"] * rq["len_in"])
    assert math.isclose(S.moe_lambda_ep(ca[0], ca[1], tokens), O.lambda_ep(cl, mo, tokens), rel_tol=1e-12)
    assert math.isclose(S.moe_lambda_mix(ca[0], ca[1], tokens), O.lambda_mix(cl, mo, tokens), rel_tol=1e-12)
    for d in (1, 2, 8):
        for fn_c, fn_o in ((S.moe_cost_rs, O.RS), (S.moe_cost_ag, O.AG), (S.moe_cost_ar, O.AR),
                           (S.moe_cost_a2a, O.A2A)):
            assert math.isclose(fn_c(1e9, d, cl["bw_inter"]), fn_o(1e9, d, cl["bw_inter"]), rel_tol=1e-12)


def test_c_argument_validation():
    cl, mo, rq = cluster(), model(), mix()
    ca = c_args(cl, mo, rq)
    for bad in ((3, 8, 1), (4, 4, 1), (4, 8, 16), (4, 8, 3), (0, 32, 1)):
        with pytest.raises(ValueError):
            S.moe_strategy_eval(*ca, *bad)
    with pytest.raises(ValueError):
        S.moe_strategy_eval(S.MoECluster(**cluster(n_proc=6)), ca[1], ca[2], 4, 8, 1)
    with pytest.raises(ValueError):
        S.moe_strategy_select(ca[0], S.MoEModel(**model(layers=0)), ca[2])
    assert math.isnan(S.moe_cost_a2a(1.0, 0, 1.0)) and math.isnan(S.moe_cost_rs(1.0, 2, 0.0))
    best, _ = S.moe_strategy_select(S.MoECluster(**cluster(mem_bytes=1 * GB)), ca[1], ca[2])
    assert best is None
