"""CPU oracle of the MoE layer share -- TEST INFRASTRUCTURE ONLY.

Thin numpy/ctypes wrapper over `moe_oracle.c` (plain C loops, fp64
arithmetic).  Only tests, the smoke check and the benchmark's cpu_baseline leg
may import this package; the HIP library and its Python binding never do, and
this package imports nothing from them.

Arrays arrive in storage form: float32, uint16 (bf16 bit patterns) or uint8
(OCP e4m3 codes, with float32 128x128 block scales passed separately) and are
decoded exactly to float32 by the oracle's own decoders before use.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "moe_oracle.c")
_LIB = os.path.join(_DIR, "liboracle.so")
# A test that plants mistakes in a copy of the source points this at the copy's
# build; the library is then loaded as it is and never rebuilt from _SRC.
_LIB_OVERRIDE = os.environ.get("MOE_ORACLE_LIB")
_lib = None

SCORE_SOFTMAX, SCORE_SIGMOID = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP).  Returns the library path."""
    if _LIB_OVERRIDE:
        return _LIB_OVERRIDE
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def decode(a: np.ndarray) -> np.ndarray:
    """Storage array -> float32 values (exact)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.float32:
        return a
    out = np.empty(a.shape, np.float32)
    if a.dtype == np.uint16:
        _load().oracle_decode_bf16(_p(a), ctypes.c_size_t(a.size), _p(out))
    elif a.dtype == np.uint8:
        _load().oracle_decode_e4m3(_p(a), ctypes.c_size_t(a.size), _p(out))
    else:
        raise TypeError(a.dtype)
    return out


def _score_code(score_fn) -> int:
    if isinstance(score_fn, str):
        return {"softmax": SCORE_SOFTMAX, "sigmoid": SCORE_SIGMOID}[score_fn]
    return int(score_fn)


def route(x, gate_w, k, score_fn="softmax", renormalize=True, routed_scale=1.0,
          n_groups=1, topk_groups=1, group_score_n=0, logit_bias=None, select_bias=None,
          logits_in=None, return_logits=False):
    """Gate scoring + top-k.  Returns ids int32 [T,k] (pick order), w float32
    [T,k], margin float64 [T] (and the fp64 logits [T,E] on request)."""
    gate_w = decode(gate_w)
    E, H = gate_w.shape
    if logits_in is not None:
        logits_in = np.ascontiguousarray(logits_in, np.float32)
        T = logits_in.shape[0]
        xf = None
    else:
        xf = decode(x)
        T = xf.shape[0]
        assert xf.shape[1] == H
    if n_groups > 1:
        assert E % n_groups == 0 and 1 <= topk_groups <= n_groups
        assert 1 <= group_score_n <= E // n_groups
        assert k <= topk_groups * (E // n_groups)
    assert 1 <= k <= E
    lb = None if logit_bias is None else np.ascontiguousarray(logit_bias, np.float32)
    sb = None if select_bias is None else np.ascontiguousarray(select_bias, np.float32)
    ids = np.empty((T, k), np.int32)
    w = np.empty((T, k), np.float32)
    margin = np.empty((T,), np.float64)
    logits = np.empty((T, E), np.float64) if return_logits else None
    _load().oracle_route(T, H, E, k, _score_code(score_fn), int(bool(renormalize)),
                         ctypes.c_double(routed_scale), n_groups, topk_groups, group_score_n,
                         _p(xf), _p(gate_w), _p(lb), _p(sb), _p(logits_in),
                         _p(ids), _p(w), _p(margin), _p(logits))
    return (ids, w, margin, logits) if return_logits else (ids, w, margin)


def dispatch(ids, x, e_lo, e_hi, want_xs=True):
    """Expert-contiguous buffer build.  Returns counts, offsets, perm (length
    A_loc), inv [T*k], xs float32 [A_loc,H] (None when want_xs is False)."""
    ids = np.ascontiguousarray(ids, np.int32)
    T, k = ids.shape
    if not want_xs:
        E_loc = e_hi - e_lo
        counts = np.empty((E_loc,), np.int32)
        offsets = np.empty((E_loc + 1,), np.int32)
        perm = np.full((T * k,), -1, np.int32)
        inv = np.empty((T * k,), np.int32)
        _load().oracle_dispatch(T, k, 0, e_lo, e_hi, _p(ids), None, _p(counts), _p(offsets),
                                _p(perm), _p(inv), None)
        return counts, offsets, perm[:int(offsets[-1])].copy(), inv, None
    xf = decode(x)
    H = xf.shape[1]
    E_loc = e_hi - e_lo
    counts = np.empty((E_loc,), np.int32)
    offsets = np.empty((E_loc + 1,), np.int32)
    perm = np.full((T * k,), -1, np.int32)
    inv = np.empty((T * k,), np.int32)
    xs = np.zeros((T * k, H), np.float32)
    _load().oracle_dispatch(T, k, H, e_lo, e_hi, _p(ids), _p(xf), _p(counts), _p(offsets),
                            _p(perm), _p(inv), _p(xs))
    n = int(offsets[-1])
    return counts, offsets, perm[:n].copy(), inv, xs[:n].copy()


def expert_ffn(offsets, xs, w_gate, w_up, w_down, s_gate=None, s_up=None, s_down=None):
    """Grouped SwiGLU MLP over expert-contiguous rows.  Returns ys float64."""
    offsets = np.ascontiguousarray(offsets, np.int32)
    xs = decode(xs)
    wg, wu, wd = decode(w_gate), decode(w_up), decode(w_down)
    n, I, H = wg.shape
    assert wu.shape == (n, I, H) and wd.shape == (n, H, I) and offsets.shape == (n + 1,)
    assert xs.shape[1] == H and xs.shape[0] >= offsets[-1]
    sc = [None if s is None else np.ascontiguousarray(s, np.float32) for s in (s_gate, s_up, s_down)]
    ys = np.zeros((xs.shape[0], H), np.float64)
    _load().oracle_expert_ffn(n, _p(offsets), H, I, _p(xs), _p(wg), _p(wu), _p(wd),
                              _p(sc[0]), _p(sc[1]), _p(sc[2]), _p(ys))
    return ys


def quant_act_1x128(x):
    """On-the-fly activation quantisation, one scale per row and 128 columns.
    Returns (codes uint8 [rows,K], scales float32 [rows,K/128])."""
    x = decode(x)
    rows, K = x.shape
    assert K % 128 == 0
    codes = np.empty((rows, K), np.uint8)
    scales = np.empty((rows, K // 128), np.float32)
    _load().oracle_quant_act_1x128(rows, K, _p(x), _p(codes), _p(scales))
    return codes, scales


def expert_ffn_fp8act(offsets, xs, w_gate, w_up, w_down, s_gate, s_up, s_down):
    """The grouped SwiGLU MLP with activations quantised 1x128 on the fly (input
    rows, and the SwiGLU intermediate, which goes to the quantiser without any
    intermediate storage rounding) and block-scaled e4m3 weights.
    Returns ys float64."""
    offsets = np.ascontiguousarray(offsets, np.int32)
    xs = decode(xs)
    wg, wu, wd = decode(w_gate), decode(w_up), decode(w_down)
    n, I, H = wg.shape
    assert H % 128 == 0 and I % 128 == 0
    assert wu.shape == (n, I, H) and wd.shape == (n, H, I) and offsets.shape == (n + 1,)
    assert xs.shape[1] == H and xs.shape[0] >= offsets[-1]
    sc = [np.ascontiguousarray(s, np.float32) for s in (s_gate, s_up, s_down)]
    ys = np.zeros((xs.shape[0], H), np.float64)
    _load().oracle_expert_ffn_fp8act(n, _p(offsets), H, I, _p(xs), _p(wg), _p(wu), _p(wd),
                                     _p(sc[0]), _p(sc[1]), _p(sc[2]), _p(ys))
    return ys


def combine(ys, inv, w, shared_ys=None):
    """Gate-weighted return along the route.  Returns out float32 [T,H]."""
    ys = np.ascontiguousarray(ys, np.float64)
    w = np.ascontiguousarray(w, np.float32)
    T, k = w.shape
    H = ys.shape[1]
    if ys.shape[0] == 0:
        ys = np.zeros((1, H), np.float64)
    inv = np.ascontiguousarray(inv, np.int32).reshape(T * k)
    sh = None if shared_ys is None else np.ascontiguousarray(shared_ys, np.float64)
    out = np.empty((T, H), np.float32)
    _load().oracle_combine(T, k, H, _p(ys), _p(inv), _p(w), _p(sh), _p(out))
    return out


def dispatch_shard(ids, x, e_lo, e_hi, tp_rank, tp_size):
    """Send buffer of TP rank `tp_rank` of `tp_size` in the fused AG-Dispatch
    schedule: the rank's hidden-column shard of every routed row.  Returns
    counts, offsets, perm, inv, xs_shard float32 [A_loc, H/tp_size]."""
    ids = np.ascontiguousarray(ids, np.int32)
    T, k = ids.shape
    xf = decode(x)
    H = xf.shape[1]
    assert H % tp_size == 0 and 0 <= tp_rank < tp_size
    E_loc = e_hi - e_lo
    counts = np.empty((E_loc,), np.int32)
    offsets = np.empty((E_loc + 1,), np.int32)
    perm = np.full((T * k,), -1, np.int32)
    inv = np.empty((T * k,), np.int32)
    xs = np.zeros((T * k, H // tp_size), np.float32)
    _load().oracle_dispatch_shard(T, k, H, e_lo, e_hi, tp_rank, tp_size, _p(ids), _p(xf),
                                  _p(counts), _p(offsets), _p(perm), _p(inv), _p(xs))
    n = int(offsets[-1])
    return counts, offsets, perm[:n].copy(), inv, xs[:n].copy()


def combine_stage(ys_block, inv, w, out_block=None):
    """One stage of the fused RS-Combine on one hidden-column block:
    out_block (+)= gate-weighted rows of ys_block.  `out_block` None starts a
    new block (accumulate = 0); otherwise it is added to.  Returns float32."""
    ys_block = np.ascontiguousarray(ys_block, np.float64)
    w = np.ascontiguousarray(w, np.float32)
    T, k = w.shape
    Hb = ys_block.shape[1]
    if ys_block.shape[0] == 0:
        ys_block = np.zeros((1, Hb), np.float64)
    inv = np.ascontiguousarray(inv, np.int32).reshape(T * k)
    acc = 0 if out_block is None else 1
    out = np.empty((T, Hb), np.float32) if out_block is None else np.array(out_block, np.float32, order="C")
    _load().oracle_combine_stage(T, k, Hb, _p(ys_block), _p(inv), _p(w), acc, _p(out))
    return out


def layer_share(x, ids, w, e_lo, e_hi, experts, shared=None, fp8_activations=False):
    """dispatch -> expert MLP -> (shared expert) -> combine for given routing.
    `experts` / `shared` are dicts with w_gate,w_up,w_down,s_gate,s_up,s_down.
    `fp8_activations`: both MLPs quantise their activations (expert_ffn_fp8act).
    Returns (out float32 [T,H], parts dict)."""
    ffn = expert_ffn_fp8act if fp8_activations else expert_ffn
    counts, offsets, perm, inv, xs = dispatch(ids, x, e_lo, e_hi)
    ys = ffn(offsets, xs, experts["w_gate"], experts["w_up"], experts["w_down"],
             experts.get("s_gate"), experts.get("s_up"), experts.get("s_down"))
    ysh = None
    if shared is not None:
        T = ids.shape[0]
        ysh = ffn(np.array([0, T], np.int32), x, shared["w_gate"], shared["w_up"],
                  shared["w_down"], shared.get("s_gate"), shared.get("s_up"),
                  shared.get("s_down"))
    out = combine(ys, inv, w, ysh)
    return out, {"counts": counts, "offsets": offsets, "perm": perm, "inv": inv, "xs": xs,
                 "ys": ys, "shared_ys": ysh}
