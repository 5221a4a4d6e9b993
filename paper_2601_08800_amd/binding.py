"""ctypes binding of include/moe.h -- argument marshalling only."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

MOE_OK, MOE_ERR_INVALID_ARG, MOE_ERR_UNSUPPORTED, MOE_ERR_WORKSPACE, MOE_ERR_DEVICE = range(5)
MOE_F32, MOE_BF16, MOE_FP8_E4M3_B128 = 0, 1, 2
MOE_SCORE_SOFTMAX, MOE_SCORE_SIGMOID = 0, 1

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libmoe.so")
_lib = None

EXPORTS = ("moe_workspace_bytes", "moe_status_string", "moe_route", "moe_dispatch",
           "moe_dispatch_noalloc", "moe_dispatch_noalloc_max_bytes",
           "moe_dispatch_shard", "moe_expert_ffn", "moe_combine", "moe_combine_stage",
           "moe_fp8act_workspace_bytes", "moe_expert_ffn_fp8act", "moe_quant_act",
           "moe_dispatch_fp8q", "moe_expert_ffn_fp8q",
           "moe_profile_enable", "moe_profile_read",
           "moe_profile_filter", "moe_probe_mfma_rate",
           "moe_kernel_name")
MOE_K_COUNT = 12


class MoEConfig(ctypes.Structure):
    """Mirror of `moe_config`."""
    _fields_ = [("hidden", ctypes.c_int32), ("n_experts", ctypes.c_int32),
                ("top_k", ctypes.c_int32), ("score_fn", ctypes.c_int32),
                ("renormalize", ctypes.c_int32), ("routed_scale", ctypes.c_float),
                ("n_groups", ctypes.c_int32), ("topk_groups", ctypes.c_int32),
                ("group_score_n", ctypes.c_int32), ("expert_lo", ctypes.c_int32),
                ("expert_hi", ctypes.c_int32), ("inter_local", ctypes.c_int32),
                ("act_dtype", ctypes.c_int32), ("weight_dtype", ctypes.c_int32)]

    @property
    def n_local(self) -> int:
        return self.expert_hi - self.expert_lo


class MoEError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, moe_status_string(status), status))


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libmoe.so (built in-tree by `build.py`).  Fails loudly when absent:
    there is no fallback path."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError("libmoe.so is not built: run `python -m paper_2601_08800_amd.build` "
                               "(or __graft_entry__.build()) first")
        lib = ctypes.CDLL(_LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        cfgp = ctypes.POINTER(MoEConfig)
        lib.moe_workspace_bytes.restype = sz
        lib.moe_workspace_bytes.argtypes = [cfgp, i32]
        lib.moe_status_string.restype = ctypes.c_char_p
        lib.moe_status_string.argtypes = [ctypes.c_int]
        lib.moe_route.restype = ctypes.c_int
        lib.moe_route.argtypes = [cfgp, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.moe_dispatch.restype = ctypes.c_int
        lib.moe_dispatch.argtypes = [cfgp, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.moe_dispatch_noalloc.restype = ctypes.c_int
        lib.moe_dispatch_noalloc.argtypes = [cfgp, i32, vp, vp, vp, vp, vp, vp, vp, vp]
        lib.moe_dispatch_noalloc_max_bytes.restype = sz
        lib.moe_dispatch_noalloc_max_bytes.argtypes = []
        lib.moe_dispatch_shard.restype = ctypes.c_int
        lib.moe_dispatch_shard.argtypes = [cfgp, i32, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.moe_combine_stage.restype = ctypes.c_int
        lib.moe_combine_stage.argtypes = [cfgp, i32, vp, vp, vp, i32, i32, vp, vp]
        lib.moe_expert_ffn.restype = ctypes.c_int
        lib.moe_expert_ffn.argtypes = [cfgp, i32, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.moe_expert_ffn_fp8act.restype = ctypes.c_int
        lib.moe_expert_ffn_fp8act.argtypes = [cfgp, i32, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.moe_quant_act.restype = ctypes.c_int
        lib.moe_quant_act.argtypes = [cfgp, i32, vp, vp, vp, vp]
        lib.moe_dispatch_fp8q.restype = ctypes.c_int
        lib.moe_dispatch_fp8q.argtypes = [cfgp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.moe_expert_ffn_fp8q.restype = ctypes.c_int
        lib.moe_expert_ffn_fp8q.argtypes = [cfgp, i32, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.moe_fp8act_workspace_bytes.restype = sz
        lib.moe_fp8act_workspace_bytes.argtypes = [cfgp, i32, i32]
        lib.moe_combine.restype = ctypes.c_int
        lib.moe_combine.argtypes = [cfgp, i32, vp, vp, vp, vp, vp, vp]
        lib.moe_profile_enable.restype = ctypes.c_int
        lib.moe_profile_enable.argtypes = [i32]
        lib.moe_profile_read.restype = ctypes.c_int
        lib.moe_profile_read.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i32)]
        lib.moe_profile_filter.restype = ctypes.c_int
        lib.moe_profile_filter.argtypes = [ctypes.c_uint32]
        lib.moe_probe_mfma_rate.restype = ctypes.c_int
        lib.moe_probe_mfma_rate.argtypes = [i32, i32, vp, ctypes.POINTER(ctypes.c_double)]
        lib.moe_kernel_name.restype = ctypes.c_char_p
        lib.moe_kernel_name.argtypes = [i32]
        _lib = lib
    return _lib


def _ptr(t) -> Optional[int]:
    """Device (or raw integer) pointer of a tensor-like; None stays NULL."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(status: int, where: str):
    if status != MOE_OK:
        raise MoEError(status, where)


def moe_status_string(status: int) -> str:
    return load_library().moe_status_string(int(status)).decode()


def moe_workspace_bytes(cfg: MoEConfig, T: int) -> int:
    return int(load_library().moe_workspace_bytes(ctypes.byref(cfg), T))


def _ws_bytes(ws) -> int:
    return 0 if ws is None else ws.numel() * ws.element_size()


def moe_route(cfg, T, x, gate_w, logit_bias, select_bias, logits_in, topk_ids, topk_w, ws,
              stream=None, ws_bytes=None):
    st = load_library().moe_route(ctypes.byref(cfg), T, _ptr(x), _ptr(gate_w), _ptr(logit_bias),
                                  _ptr(select_bias), _ptr(logits_in), _ptr(topk_ids), _ptr(topk_w),
                                  _ptr(ws), _ws_bytes(ws) if ws_bytes is None else ws_bytes,
                                  _stream(stream))
    _check(st, "moe_route")


def moe_dispatch(cfg, T, x, topk_ids, counts, offsets, perm, inv, xs, ws, stream=None,
                 ws_bytes=None):
    st = load_library().moe_dispatch(ctypes.byref(cfg), T, _ptr(x), _ptr(topk_ids), _ptr(counts),
                                     _ptr(offsets), _ptr(perm), _ptr(inv), _ptr(xs), _ptr(ws),
                                     _ws_bytes(ws) if ws_bytes is None else ws_bytes,
                                     _stream(stream))
    _check(st, "moe_dispatch")


def moe_dispatch_noalloc_max_bytes() -> int:
    return int(load_library().moe_dispatch_noalloc_max_bytes())


def moe_dispatch_noalloc(cfg, T, x, topk_ids, counts, offsets, perm, inv, xs, stream=None):
    st = load_library().moe_dispatch_noalloc(ctypes.byref(cfg), T, _ptr(x), _ptr(topk_ids),
                                             _ptr(counts), _ptr(offsets), _ptr(perm), _ptr(inv),
                                             _ptr(xs), _stream(stream))
    _check(st, "moe_dispatch_noalloc")


def moe_dispatch_shard(cfg, T, x, topk_ids, tp_rank, tp_size, counts, offsets, perm, inv, xs_shard,
                       ws, stream=None, ws_bytes=None):
    st = load_library().moe_dispatch_shard(ctypes.byref(cfg), T, _ptr(x), _ptr(topk_ids), tp_rank,
                                           tp_size, _ptr(counts), _ptr(offsets), _ptr(perm),
                                           _ptr(inv), _ptr(xs_shard), _ptr(ws),
                                           _ws_bytes(ws) if ws_bytes is None else ws_bytes,
                                           _stream(stream))
    _check(st, "moe_dispatch_shard")


def moe_expert_ffn(cfg, n_experts_here, xs, offsets, rows_capacity, w_gate, w_up, w_down,
                   s_gate, s_up, s_down, ys, ws, stream=None, ws_bytes=None):
    st = load_library().moe_expert_ffn(ctypes.byref(cfg), n_experts_here, _ptr(xs), _ptr(offsets),
                                       rows_capacity, _ptr(w_gate), _ptr(w_up), _ptr(w_down),
                                       _ptr(s_gate), _ptr(s_up), _ptr(s_down), _ptr(ys), _ptr(ws),
                                       _ws_bytes(ws) if ws_bytes is None else ws_bytes,
                                       _stream(stream))
    _check(st, "moe_expert_ffn")


def moe_fp8act_workspace_bytes(cfg: MoEConfig, n_experts_here: int, rows_capacity: int) -> int:
    return int(load_library().moe_fp8act_workspace_bytes(ctypes.byref(cfg), n_experts_here, rows_capacity))


def moe_expert_ffn_fp8act(cfg, n_experts_here, xs, offsets, rows_capacity, w_gate, w_up, w_down,
                          s_gate, s_up, s_down, ys, ws, stream=None, ws_bytes=None):
    st = load_library().moe_expert_ffn_fp8act(
        ctypes.byref(cfg), n_experts_here, _ptr(xs), _ptr(offsets), rows_capacity, _ptr(w_gate),
        _ptr(w_up), _ptr(w_down), _ptr(s_gate), _ptr(s_up), _ptr(s_down), _ptr(ys), _ptr(ws),
        _ws_bytes(ws) if ws_bytes is None else ws_bytes, _stream(stream))
    _check(st, "moe_expert_ffn_fp8act")


def moe_quant_act(cfg, rows, x, codes, scales, stream=None):
    st = load_library().moe_quant_act(ctypes.byref(cfg), rows, _ptr(x), _ptr(codes), _ptr(scales),
                                      _stream(stream))
    _check(st, "moe_quant_act")


def moe_dispatch_fp8q(cfg, T, xq, xq_scales, topk_ids, counts, offsets, perm, inv, xs_q, xs_scales,
                      ws, stream=None, ws_bytes=None):
    st = load_library().moe_dispatch_fp8q(
        ctypes.byref(cfg), T, _ptr(xq), _ptr(xq_scales), _ptr(topk_ids), _ptr(counts), _ptr(offsets),
        _ptr(perm), _ptr(inv), _ptr(xs_q), _ptr(xs_scales), _ptr(ws),
        _ws_bytes(ws) if ws_bytes is None else ws_bytes, _stream(stream))
    _check(st, "moe_dispatch_fp8q")


def moe_expert_ffn_fp8q(cfg, n_experts_here, xs_q, xs_scales, offsets, rows_capacity, w_gate, w_up,
                        w_down, s_gate, s_up, s_down, ys, ws, stream=None, ws_bytes=None):
    st = load_library().moe_expert_ffn_fp8q(
        ctypes.byref(cfg), n_experts_here, _ptr(xs_q), _ptr(xs_scales), _ptr(offsets), rows_capacity,
        _ptr(w_gate), _ptr(w_up), _ptr(w_down), _ptr(s_gate), _ptr(s_up), _ptr(s_down), _ptr(ys),
        _ptr(ws), _ws_bytes(ws) if ws_bytes is None else ws_bytes, _stream(stream))
    _check(st, "moe_expert_ffn_fp8q")


def moe_combine(cfg, T, ys, inv, topk_w, shared_ys, out, stream=None):
    st = load_library().moe_combine(ctypes.byref(cfg), T, _ptr(ys), _ptr(inv), _ptr(topk_w),
                                    _ptr(shared_ys), _ptr(out), _stream(stream))
    _check(st, "moe_combine")


def moe_combine_stage(cfg, T, ys_block, inv, topk_w, tp_size, accumulate, out_block, stream=None):
    st = load_library().moe_combine_stage(ctypes.byref(cfg), T, _ptr(ys_block), _ptr(inv),
                                          _ptr(topk_w), tp_size, int(accumulate), _ptr(out_block),
                                          _stream(stream))
    _check(st, "moe_combine_stage")


def moe_profile_enable(max_records: int):
    _check(load_library().moe_profile_enable(max_records), "moe_profile_enable")


def moe_probe_mfma_rate(workgroups: int, iters: int, stream=None) -> float:
    """TFLOP/s of a register-only bf16 MFMA loop on this machine (calibration)."""
    out = ctypes.c_double(0.0)
    _check(load_library().moe_probe_mfma_rate(workgroups, iters, _stream(stream), ctypes.byref(out)),
           "moe_probe_mfma_rate")
    return out.value


def moe_profile_filter(names=None):
    """Record only the named kernels (None: all)."""
    lib = load_library()
    mask = 0xffffffff
    if names is not None:
        ids = {lib.moe_kernel_name(i).decode(): i for i in range(MOE_K_COUNT)}
        mask = 0
        for n in names:
            mask |= 1 << ids[n]
    _check(lib.moe_profile_filter(mask), "moe_profile_filter")


def moe_profile_read():
    """{kernel name: (total ms, launches)} of the launches recorded since the last read."""
    lib = load_library()
    ms = (ctypes.c_double * MOE_K_COUNT)()
    n = (ctypes.c_int32 * MOE_K_COUNT)()
    _check(lib.moe_profile_read(ms, n), "moe_profile_read")
    return {lib.moe_kernel_name(i).decode(): (ms[i], n[i]) for i in range(MOE_K_COUNT) if n[i]}
