"""ctypes binding of include/moe_strategy.h -- argument marshalling only."""
from __future__ import annotations

import ctypes

from .binding import load_library

STRATEGY_EXPORTS = ("moe_cost_rs", "moe_cost_ag", "moe_cost_ar", "moe_cost_a2a", "moe_lambda_ep",
                    "moe_lambda_mix", "moe_strategy_eval", "moe_strategy_select")

_i32, _f64 = ctypes.c_int32, ctypes.c_double


class MoECluster(ctypes.Structure):
    """Mirror of `moe_cluster`."""
    _fields_ = [("n_node", _i32), ("n_proc", _i32), ("mem_bytes", _f64), ("bw_intra", _f64),
                ("bw_inter", _f64), ("bw_p2p", _f64), ("compute_rate", _f64)]


class MoEModel(ctypes.Structure):
    """Mirror of `moe_model`."""
    _fields_ = [("psi_attn", _f64), ("psi_moe", _f64), ("layers", _i32), ("hidden", _i32),
                ("top_k", _i32), ("act_bytes", _f64)]


class MoERequestMix(ctypes.Structure):
    """Mirror of `moe_request_mix`."""
    _fields_ = [("batch", _i32), ("len_in", _i32), ("len_out", _i32), ("arrival_rate", _f64),
                ("max_ttft", _f64), ("max_itl", _f64)]


class MoEStrategy(ctypes.Structure):
    """Mirror of `moe_strategy`."""
    _fields_ = [("d_tp", _i32), ("d_ep", _i32), ("d_dp", _i32), ("d_pp", _i32),
                ("tau_prf", _f64), ("lambda_prf", _f64), ("tau_dec", _f64), ("lambda_dec", _f64),
                ("svc_prf", _f64), ("svc_dec", _f64), ("wq", _f64), ("ttft", _f64), ("itl", _f64),
                ("throughput", _f64), ("mem_bytes", _f64), ("feasible", _i32)]

    def as_dict(self) -> dict:
        return {n: getattr(self, n) for n, _ in self._fields_}


_ready = False


def _lib():
    global _ready
    lib = load_library()
    if not _ready:
        for n in ("moe_cost_rs", "moe_cost_ag", "moe_cost_ar", "moe_cost_a2a"):
            getattr(lib, n).restype = _f64
            getattr(lib, n).argtypes = [_f64, _i32, _f64]
        cp, mp = ctypes.POINTER(MoECluster), ctypes.POINTER(MoEModel)
        rp, sp = ctypes.POINTER(MoERequestMix), ctypes.POINTER(MoEStrategy)
        for n in ("moe_lambda_ep", "moe_lambda_mix"):
            getattr(lib, n).restype = _f64
            getattr(lib, n).argtypes = [cp, mp, _f64]
        lib.moe_strategy_eval.restype = _i32
        lib.moe_strategy_eval.argtypes = [cp, mp, rp, _i32, _i32, _i32, _i32, sp]
        lib.moe_strategy_select.restype = _i32
        lib.moe_strategy_select.argtypes = [cp, mp, rp, _i32, sp, sp, _i32, ctypes.POINTER(_i32)]
        _ready = True
    return lib


def moe_cost_rs(size, degree, bw): return _lib().moe_cost_rs(size, degree, bw)
def moe_cost_ag(size, degree, bw): return _lib().moe_cost_ag(size, degree, bw)
def moe_cost_ar(size, degree, bw): return _lib().moe_cost_ar(size, degree, bw)
def moe_cost_a2a(size, degree, bw): return _lib().moe_cost_a2a(size, degree, bw)


def moe_lambda_ep(cluster: MoECluster, model: MoEModel, tokens: float) -> float:
    return _lib().moe_lambda_ep(ctypes.byref(cluster), ctypes.byref(model), tokens)


def moe_lambda_mix(cluster: MoECluster, model: MoEModel, tokens: float) -> float:
    return _lib().moe_lambda_mix(ctypes.byref(cluster), ctypes.byref(model), tokens)


def moe_strategy_eval(cluster, model, mix, d_tp, d_ep, d_dp, d_pp=1) -> MoEStrategy:
    out = MoEStrategy()
    rc = _lib().moe_strategy_eval(ctypes.byref(cluster), ctypes.byref(model), ctypes.byref(mix),
                                  d_tp, d_ep, d_dp, d_pp, ctypes.byref(out))
    if rc:
        raise ValueError("moe_strategy_eval: invalid arguments")
    return out


def moe_strategy_select(cluster, model, mix, d_pp=1, max_all=256):
    """Returns (best or None, list of every evaluated strategy)."""
    best = MoEStrategy()
    buf = (MoEStrategy * max_all)()
    n = _i32(0)
    rc = _lib().moe_strategy_select(ctypes.byref(cluster), ctypes.byref(model), ctypes.byref(mix),
                                    d_pp, ctypes.byref(best), buf, max_all, ctypes.byref(n))
    if rc == 1:
        raise ValueError("moe_strategy_select: invalid arguments")
    return (best if rc == 0 else None), [buf[i] for i in range(min(n.value, max_all))]
