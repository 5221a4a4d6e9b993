"""Seeded synthetic MoE-layer workloads (inputs only).

This module draws the tensors that both the CPU oracle and the HIP library are
fed with: activations, gate weights, routing biases, expert weights, and (for
the forced-routing stress case) expert assignments.  It holds storage-format
encoders (fp32 -> bf16 bits, fp32 -> OCP e4m3 codes with 128x128 block scales)
because the stored bits *are* the model; it holds none of the layer's
arithmetic (no gate scoring, top-k, dispatch, FFN or combine).

Every tensor has its own Philox stream keyed by (seed, tensor id), so any
subset can be drawn in any order and always has the same bits.

Storage conventions of the returned numpy arrays
  f32   -> float32
  bf16  -> uint16 holding the upper 16 bits of the fp32 pattern (RNE rounded)
  fp8   -> uint8 OCP e4m3 codes + float32 scales, one per 128x128 block
"""
from __future__ import annotations

import dataclasses
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np

FP8_BLOCK = 128
E4M3_MAX = 448.0

# tensor kinds for the Philox stream id
_K_X, _K_WG, _K_LBIAS, _K_SBIAS, _K_GATE, _K_UP, _K_DOWN, _K_ZIPF_G, _K_ZIPF_P, _K_ZIPF_W = range(10)
_SHARED_EXPERT_ID = 1 << 20


@dataclass(frozen=True)
class Workload:
    name: str
    seed: int
    T: int                  # tokens
    H: int                  # hidden
    E: int                  # global routed experts
    k: int                  # experts per token
    I: int                  # full expert intermediate size
    score_fn: str = "softmax"        # "softmax" | "sigmoid"
    renormalize: bool = True
    routed_scale: float = 1.0
    n_groups: int = 1
    topk_groups: int = 1
    group_score_n: int = 0
    expert_lo: int = 0
    expert_hi: int = 0               # 0 -> E
    tp: int = 1
    tp_rank: int = 0
    act_dtype: str = "bf16"          # "f32" | "bf16"
    weight_dtype: str = "bf16"       # "f32" | "bf16" | "fp8"
    shared_expert: bool = False
    x_std: float = 1.0
    w_std: float = 0.02
    logit_bias_std: float = 0.0
    select_bias_std: float = 0.0
    fp8_activations: bool = False    # expert FFN quantises its activations 1x128 to e4m3 on the fly
    zipf_s: Optional[float] = None   # forced Zipf routing exponent, or None
    zipf_perm_stream: int = 0        # which seeded rank->expert permutation is used

    @property
    def e_hi(self) -> int:
        return self.expert_hi if self.expert_hi > 0 else self.E

    @property
    def E_loc(self) -> int:
        return self.e_hi - self.expert_lo

    @property
    def I_loc(self) -> int:
        return self.I // self.tp

    def replace(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


# The shapes of the benchmark table: tiny fp32, Qwen3-30B-A3B full layer
# (prefill / decode), Qwen3-235B EP=8 share (prefill / decode), DeepSeek-R1
# TP=2 x 32-expert share (prefill), and the same share with fp8 weights under
# forced Zipf routing.
CONFIGS: Dict[str, Workload] = {
    "c1": Workload("c1", 1001, T=64, H=256, E=8, k=2, I=512, act_dtype="f32",
                   weight_dtype="f32", x_std=0.02),
    "c2p": Workload("c2p", 1002, T=4096, H=2048, E=128, k=8, I=768),
    "c2d": Workload("c2d", 1002, T=64, H=2048, E=128, k=8, I=768),
    # the largest step the paper's serving limits allow (evaluation set-up: at most
    # 16 sequences of at most 4096 tokens): send and return buffers above 2 GiB
    "c2x": Workload("c2x", 1002, T=65536, H=2048, E=128, k=8, I=768),
    "c3": Workload("c3", 1003, T=8192, H=4096, E=128, k=8, I=1536,
                   expert_lo=0, expert_hi=16, logit_bias_std=0.5),
    # the same EP=8 share at a decode batch (256 tokens in flight)
    "c3d": Workload("c3d", 1003, T=256, H=4096, E=128, k=8, I=1536,
                    expert_lo=0, expert_hi=16, logit_bias_std=0.5),
    "c4": Workload("c4", 1004, T=16384, H=7168, E=256, k=8, I=2048,
                   score_fn="sigmoid", routed_scale=2.5, n_groups=8, topk_groups=4,
                   group_score_n=2, expert_lo=0, expert_hi=32, tp=2, tp_rank=0,
                   shared_expert=True, select_bias_std=0.05),
    # the C4 share with e4m3 block-scaled weights (bf16 activations)
    "c4w": Workload("c4w", 1004, T=16384, H=7168, E=256, k=8, I=2048,
                    score_fn="sigmoid", routed_scale=2.5, n_groups=8, topk_groups=4,
                    group_score_n=2, expert_lo=0, expert_hi=32, tp=2, tp_rank=0,
                    shared_expert=True, select_bias_std=0.05, weight_dtype="fp8"),
    # the C4 share with e4m3 weights and 8-bit activations in the expert FFN
    "c4q": Workload("c4q", 1004, T=16384, H=7168, E=256, k=8, I=2048,
                    score_fn="sigmoid", routed_scale=2.5, n_groups=8, topk_groups=4,
                    group_score_n=2, expert_lo=0, expert_hi=32, tp=2, tp_rank=0,
                    shared_expert=True, select_bias_std=0.05, weight_dtype="fp8",
                    fp8_activations=True),
    "c5": Workload("c5", 1005, T=256, H=7168, E=256, k=8, I=2048,
                   score_fn="sigmoid", routed_scale=2.5, n_groups=8, topk_groups=4,
                   group_score_n=2, expert_lo=0, expert_hi=32, tp=2, tp_rank=0,
                   shared_expert=True, select_bias_std=0.05, weight_dtype="fp8",
                   # stream 11 is the first whose permutation puts two of the five
                   # hottest ranks (1 and 3) on local experts, so the skew is felt
                   zipf_s=1.2, zipf_perm_stream=11),
}


# --------------------------------------------------------------------------
# storage encoders
# --------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even); returns the 16-bit patterns.
    Inputs are finite by construction."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def f32_to_e4m3_codes(v: np.ndarray) -> np.ndarray:
    """Encode fp32 to OCP e4m3 (1-4-3, bias 7, no infinities, max 448) with
    round-to-nearest-even and saturation.  Returns uint8 codes."""
    v = np.asarray(v, dtype=np.float32)
    sign = (np.signbit(v)).astype(np.uint8) << 7
    a = np.minimum(np.abs(v).astype(np.float64), E4M3_MAX)
    # exponent of the quantum: normals 2^(e-3) with e>=-6, subnormals 2^-9
    e = np.floor(np.log2(np.maximum(a, 2.0 ** -6)))
    e = np.clip(e, -6, 8)
    quantum = np.exp2(e - 3)
    q = np.rint(a / quantum)           # RNE on exact binary fractions
    # q in [0,16]; 16 means the mantissa carried into the next binade
    carry = q >= 16
    e = np.where(carry, e + 1, e)
    q = np.where(carry, 8, q)
    is_sub = q < 8                     # below the smallest normal
    exp_field = np.where(is_sub, 0, e + 7).astype(np.int64)
    man_field = np.where(is_sub, q, q - 8).astype(np.int64)
    code = (exp_field << 3) | man_field
    code = np.minimum(code, 0x7E)      # 0x7F is NaN; saturate at 448
    return (code.astype(np.uint8) | sign).astype(np.uint8)


def quantize_e4m3_block128(w: np.ndarray):
    """Per 128x128 block: scale = max|w|/448 (fp32), codes = e4m3(w/scale)."""
    R, C = w.shape
    nr, nc = -(-R // FP8_BLOCK), -(-C // FP8_BLOCK)
    pad = np.zeros((nr * FP8_BLOCK, nc * FP8_BLOCK), np.float32)
    pad[:R, :C] = w
    blk = pad.reshape(nr, FP8_BLOCK, nc, FP8_BLOCK)
    m = np.abs(blk).max(axis=(1, 3)).astype(np.float32)
    scales = np.where(m > 0, m / np.float32(E4M3_MAX), np.float32(1.0)).astype(np.float32)
    q = (blk / scales[:, None, :, None]).astype(np.float32)
    codes = f32_to_e4m3_codes(q.reshape(nr * FP8_BLOCK, nc * FP8_BLOCK))[:R, :C]
    return np.ascontiguousarray(codes), scales


def _rng(seed: int, kind: int, idx: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed, (kind << 40) | idx]))


def _normal(seed, kind, idx, shape, std) -> np.ndarray:
    g = _rng(seed, kind, idx)
    n = int(np.prod(shape))
    a = g.standard_normal(n, dtype=np.float32)
    a *= np.float32(std)
    return a.reshape(shape)


def _store(a: np.ndarray, dtype: str):
    if dtype == "f32":
        return a
    if dtype == "bf16":
        return f32_to_bf16_bits(a)
    raise ValueError(dtype)


# --------------------------------------------------------------------------
# tensors
# --------------------------------------------------------------------------
def make_x(w: Workload) -> np.ndarray:
    """Activations [T,H] ~ N(0, x_std) in the activation storage dtype."""
    return _store(_normal(w.seed, _K_X, 0, (w.T, w.H), w.x_std), w.act_dtype)


def make_gate(w: Workload) -> dict:
    """Gate weights [E,H] ~ N(0, 1/sqrt(H)) in the activation dtype and the
    optional fp32 biases (logit bias for load skew, selection bias for the
    bias-corrected sigmoid gate)."""
    out = {"gate_w": _store(_normal(w.seed, _K_WG, 0, (w.E, w.H), 1.0 / np.sqrt(w.H)), w.act_dtype),
           "logit_bias": None, "select_bias": None}
    if w.logit_bias_std > 0:
        out["logit_bias"] = _normal(w.seed, _K_LBIAS, 0, (w.E,), w.logit_bias_std)
    if w.select_bias_std > 0:
        out["select_bias"] = _normal(w.seed, _K_SBIAS, 0, (w.E,), w.select_bias_std)
    return out


def _expert_matrix(w: Workload, kind: int, expert_id: int, tp_rank: int, shape):
    idx = (expert_id << 8) | tp_rank
    a = _normal(w.seed, kind, idx, shape, w.w_std)
    if w.weight_dtype == "fp8":
        return quantize_e4m3_block128(a)
    return _store(a, w.weight_dtype), None


def make_expert_weights(w: Workload, expert_ids, tp_rank: Optional[int] = None) -> dict:
    """TP slice `tp_rank` of the SwiGLU weights of the listed (global) expert
    ids: w_gate,w_up [n,I_loc,H]; w_down [n,H,I_loc]; block scales (fp8) or None.
    The full-I weights are by definition the concatenation of the slices."""
    tp_rank = w.tp_rank if tp_rank is None else tp_rank
    n, Il, H = len(expert_ids), w.I_loc, w.H
    wd = {"f32": np.float32, "bf16": np.uint16, "fp8": np.uint8}[w.weight_dtype]
    out = {"w_gate": np.empty((n, Il, H), wd), "w_up": np.empty((n, Il, H), wd),
           "w_down": np.empty((n, H, Il), wd), "s_gate": None, "s_up": None, "s_down": None}
    if w.weight_dtype == "fp8":
        bi, bh = -(-Il // FP8_BLOCK), -(-H // FP8_BLOCK)
        out["s_gate"] = np.empty((n, bi, bh), np.float32)
        out["s_up"] = np.empty((n, bi, bh), np.float32)
        out["s_down"] = np.empty((n, bh, bi), np.float32)
    jobs = [(i, int(e), name, sname, kind, shape)
            for i, e in enumerate(expert_ids)
            for name, sname, kind, shape in (("w_gate", "s_gate", _K_GATE, (Il, H)),
                                             ("w_up", "s_up", _K_UP, (Il, H)),
                                             ("w_down", "s_down", _K_DOWN, (H, Il)))]

    def run(job):
        i, e, name, sname, kind, shape = job
        q, s = _expert_matrix(w, kind, e, tp_rank, shape)
        out[name][i] = q
        if s is not None:
            out[sname][i] = s

    if len(jobs) > 3:       # independent streams: draw them on a few threads
        with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
            list(ex.map(run, jobs))
    else:
        for j in jobs:
            run(j)
    return out


def make_local_experts(w: Workload, tp_rank: Optional[int] = None) -> dict:
    return make_expert_weights(w, range(w.expert_lo, w.e_hi), tp_rank)


def make_shared_expert(w: Workload, tp_rank: Optional[int] = None) -> dict:
    return make_expert_weights(w, [_SHARED_EXPERT_ID], tp_rank)


def make_forced_routing(w: Workload):
    """Forced Zipf-skewed routing: per token k distinct experts drawn with
    probability proportional to rank^-s (Gumbel top-k), rank -> expert through
    a seeded permutation; weights are seeded positive numbers normalised to
    routed_scale.  Returns (topk_ids int32 [T,k], topk_w float32 [T,k])."""
    assert w.zipf_s is not None
    ranks = np.arange(1, w.E + 1, dtype=np.float64)
    logp = -w.zipf_s * np.log(ranks)
    g = _rng(w.seed, _K_ZIPF_G).gumbel(size=(w.T, w.E))
    perm = _rng(w.seed, _K_ZIPF_P, w.zipf_perm_stream).permutation(w.E)        # rank index -> expert id
    top = np.argsort(-(logp[None, :] + g), axis=1, kind="stable")[:, : w.k]
    ids = perm[top].astype(np.int32)
    z = _rng(w.seed, _K_ZIPF_W).standard_normal((w.T, w.k))
    s = 1.0 / (1.0 + np.exp(-z))
    wts = (s / s.sum(axis=1, keepdims=True) * w.routed_scale).astype(np.float32)
    return ids, wts
