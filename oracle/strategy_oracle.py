"""Reference for the analytic strategy selector: the latency model of Sec. III-A
and the enumeration of Sec. III-B-2 written out equation by equation in plain
Python floats.  TEST INFRASTRUCTURE ONLY: imported by tests, never by the
product path, and shares no code with the C implementation.

Constants of proportionality: a collective over a group moves at `bw` bytes/s
(bw_intra when the group fits into a node, else bw_inter); the compute term is
divided by `compute_rate`.  Readings of the paper taken here (the same list is in
the design notes): a group of one device costs nothing; AR is taken as printed,
RS and AG of size/degree; Psi in the compute term is the weights of ONE layer
(the service latency multiplies by l); the queue's service rate is the decode
(s = 1) per-token rate; the K/V term of the memory constraint uses the longest
context L_in + L_out.
"""
import math


def RS(size, degree, bw):
    """Sec. III-A-2, first equation: RS = AG ~ size / degree."""
    return 0.0 if degree == 1 else size / degree / bw


AG = RS


def AR(size, degree, bw):
    """Second equation: AR(size, d) = RS(size/d, d) + AG(size/d, d)."""
    return RS(size / degree, degree, bw) + AG(size / degree, degree, bw)


def A2A(size, degree, bw):
    """Third equation: A2A ~ size / degree * (degree - 1)."""
    return size / degree * (degree - 1) / bw


def _bw(cl, devices):
    return cl["bw_intra"] if devices <= cl["n_proc"] else cl["bw_inter"]


def tau(cl, mo, b, s, d_tp, d_ep, d_dp):
    """Computational latency of a layer: Psi / (d_TP d_EP) * b / d_DP * s h."""
    psi = (mo["psi_attn"] + mo["psi_moe"]) / mo["layers"]
    return psi / (d_tp * d_ep) * (b / d_dp) * s * mo["hidden"] / cl["compute_rate"]


def lam(cl, mo, b, s, d_tp, d_ep, d_dp):
    """Communication latency of a layer: 2 AR(b/d_DP sh, d_TP) + 2 A2A(...), with
    the A2A running in groups of d_EP devices on b/d_DP sequences when d_DP >=
    d_EP, else in groups of d_DP devices on b/d_EP sequences."""
    h, k, eb = mo["hidden"], mo["top_k"], mo["act_bytes"]
    ar = AR(b / d_dp * s * h * eb, d_tp, _bw(cl, d_tp))
    if d_dp >= d_ep:
        a2a = A2A(b / d_dp * s * h * k * eb, d_ep, _bw(cl, d_tp * d_ep))
    else:
        a2a = A2A(b / d_ep * s * h * k * eb, d_dp, _bw(cl, d_tp * d_dp))
    return 2 * ar + 2 * a2a


def service(cl, mo, b, s, d_tp, d_ep, d_dp, d_pp):
    """l [tau + lambda] + (d_PP - 1) P2P(b/d_DP sh)."""
    p2p = b / d_dp * s * mo["hidden"] * mo["act_bytes"] / cl["bw_p2p"]
    return mo["layers"] * (tau(cl, mo, b, s, d_tp, d_ep, d_dp) + lam(cl, mo, b, s, d_tp, d_ep, d_dp)) \
        + (d_pp - 1) * p2p


def evaluate(cl, mo, rq, d_tp, d_ep, d_dp, d_pp):
    b, L_in, L_out = rq["batch"], rq["len_in"], rq["len_out"]
    out = dict(d_tp=d_tp, d_ep=d_ep, d_dp=d_dp, d_pp=d_pp)
    out["tau_prf"] = tau(cl, mo, b, L_in, d_tp, d_ep, d_dp)
    out["lambda_prf"] = lam(cl, mo, b, L_in, d_tp, d_ep, d_dp)
    out["tau_dec"] = tau(cl, mo, b, 1, d_tp, d_ep, d_dp)
    out["lambda_dec"] = lam(cl, mo, b, 1, d_tp, d_ep, d_dp)
    out["svc_prf"] = service(cl, mo, b, L_in, d_tp, d_ep, d_dp, d_pp)
    out["svc_dec"] = service(cl, mo, b, 1, d_tp, d_ep, d_dp, d_pp)
    mu = 1.0 / out["svc_dec"]
    la = rq["arrival_rate"]
    if la == 0:
        wq = 0.0
    elif la < mu:
        rho = la / mu
        wq = rho / (mu * (1 - rho))          # = la / (mu (mu - la))
    else:
        wq = math.inf
    out["wq"] = wq
    out["ttft"] = wq + out["svc_prf"]
    out["itl"] = out["svc_dec"]
    out["throughput"] = (L_in + L_out) / (wq + out["svc_prf"] + L_out * out["svc_dec"])
    out["mem_bytes"] = mo["psi_attn"] / d_tp + mo["psi_moe"] / (d_ep * d_tp) \
        + 2 * b * (L_in + L_out) * mo["hidden"] * mo["act_bytes"] * mo["layers"] / d_pp
    out["feasible"] = int(out["mem_bytes"] < cl["mem_bytes"] and math.isfinite(wq)
                          and (rq["max_ttft"] == 0 or out["ttft"] <= rq["max_ttft"])
                          and (rq["max_itl"] == 0 or out["itl"] <= rq["max_itl"]))
    return out


def enumerate_strategies(cl, mo, rq, d_pp):
    """All (d_TP, d_EP, d_DP) with d_TP d_EP = n_proc n_node (Sec. III-B-2), powers
    of two, d_DP d_TP <= devices, d_DP <= b."""
    n = cl["n_node"] * cl["n_proc"]
    res = []
    d_tp = 1
    while d_tp <= n:
        d_dp = 1
        while d_dp * d_tp <= n and d_dp <= rq["batch"]:
            res.append(evaluate(cl, mo, rq, d_tp, n // d_tp, d_dp, d_pp))
            d_dp *= 2
        d_tp *= 2
    return res


def select(cl, mo, rq, d_pp):
    """The feasible strategy of largest throughput (ties: smaller ITL, smaller
    d_TP, larger d_DP); None when nothing is feasible."""
    cand = [s for s in enumerate_strategies(cl, mo, rq, d_pp) if s["feasible"]]
    if not cand:
        return None
    return min(cand, key=lambda s: (-s["throughput"], s["itl"], s["d_tp"], -s["d_dp"]))


def lambda_ep(cl, mo, tokens):
    """Pure EP in the MoE block: AR(bsh, n_proc) + 2 A2A(bshk, n_node)."""
    bsh = tokens * mo["hidden"] * mo["act_bytes"]
    return AR(bsh, cl["n_proc"], cl["bw_intra"]) + 2 * A2A(bsh * mo["top_k"], cl["n_node"], cl["bw_inter"])


def lambda_mix(cl, mo, tokens):
    """Hybrid TP-EP: AR(bsh, n_proc) + AG(bshk/n_proc, n_proc) + 2 A2A(bshk/n_proc, n_node)."""
    bsh = tokens * mo["hidden"] * mo["act_bytes"]
    sh = bsh * mo["top_k"] / cl["n_proc"]
    return AR(bsh, cl["n_proc"], cl["bw_intra"]) + AG(sh, cl["n_proc"], cl["bw_intra"]) \
        + 2 * A2A(sh, cl["n_node"], cl["bw_inter"])
