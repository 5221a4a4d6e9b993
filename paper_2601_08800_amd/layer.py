"""Buffer plumbing for one layer share: allocates the device buffers once
(torch is the allocator) and chains the four library calls on one stream.
No arithmetic happens here."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B

_ACT = {"f32": B.MOE_F32, "bf16": B.MOE_BF16}
_WT = {"f32": B.MOE_F32, "bf16": B.MOE_BF16, "fp8": B.MOE_FP8_E4M3_B128}
_SCORE = {"softmax": B.MOE_SCORE_SOFTMAX, "sigmoid": B.MOE_SCORE_SIGMOID}


def config_from_workload(w) -> B.MoEConfig:
    """moe_config for a `workloads.gen.Workload`-like object."""
    return B.MoEConfig(hidden=w.H, n_experts=w.E, top_k=w.k, score_fn=_SCORE[w.score_fn],
                       renormalize=int(w.renormalize), routed_scale=float(w.routed_scale),
                       n_groups=w.n_groups, topk_groups=w.topk_groups,
                       group_score_n=w.group_score_n, expert_lo=w.expert_lo, expert_hi=w.e_hi,
                       inter_local=w.I_loc, act_dtype=_ACT[w.act_dtype],
                       weight_dtype=_WT[w.weight_dtype])


def to_device(a, device="cuda"):
    """numpy storage array -> device tensor with the same bits (uint16 -> bf16,
    uint8 -> uint8 codes)."""
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a))
    if a.dtype == np.uint16:
        t = t.view(torch.bfloat16)
    return t.to(device)


class MoELayerShare:
    """Holds the resident inputs and every intermediate / output buffer of one
    GPU's share; `forward()` enqueues route, dispatch, expert FFN (+ shared
    expert) and combine."""

    def __init__(self, cfg: B.MoEConfig, T: int, gate, experts, shared=None, device="cuda",
                 fp8_activations: bool = False):
        self.cfg, self.T, self.dev = cfg, T, device
        # both FFN calls go through moe_expert_ffn_fp8act (e4m3 weights required)
        self.fp8_activations = fp8_activations
        k, H, El = cfg.top_k, cfg.hidden, cfg.n_local
        adt = torch.float32 if cfg.act_dtype == B.MOE_F32 else torch.bfloat16
        self.gate = {n: to_device(v, device) for n, v in gate.items()}
        self.experts = {n: to_device(v, device) for n, v in experts.items()}
        self.shared = None if shared is None else {n: to_device(v, device) for n, v in shared.items()}
        A = T * k
        e = lambda *s, dt=torch.int32: torch.empty(*s, dtype=dt, device=device)
        self.topk_ids, self.topk_w = e(T, k), e(T, k, dt=torch.float32)
        self.counts, self.offsets = e(El), e(El + 1)
        self.perm, self.inv = e(A), e(A)
        self.xs, self.ys = e(A, H, dt=adt), e(A, H, dt=adt)
        self.out = e(T, H, dt=torch.float32)
        ws_bytes = B.moe_workspace_bytes(cfg, T)
        if fp8_activations:
            need = max(B.moe_fp8act_workspace_bytes(cfg, El, A), B.moe_fp8act_workspace_bytes(cfg, 1, T))
            if need == 0:
                raise ValueError("fp8 activations need bf16 activations, e4m3 weights and sizes that are multiples of 128")
            ws_bytes = max(ws_bytes, need)
        self.ws = e(max(ws_bytes, 256), dt=torch.uint8)
        if fp8_activations:      # a token is quantised once; dispatch copies the 1-byte codes
            self.xq, self.xq_scales = e(T, H, dt=torch.uint8), e(H // 128, T, dt=torch.float32)
            self.xs_q, self.xs_scales = e(A, H, dt=torch.uint8), e(H // 128, A, dt=torch.float32)
        self.shared_ys = None
        # The shared expert depends on x only, not on the routing: by default it is
        # enqueued on a second stream (default priority) with a workspace of its own,
        # so its GEMMs fill the CUs that the routing kernels and the tail of the
        # routed GEMMs leave idle; combine waits for both streams.
        self.overlap_shared = False
        if self.shared is not None:
            self.shared_ys = e(T, H, dt=adt)
            self.shared_offsets = torch.tensor([0, T], dtype=torch.int32, device=device)
            if torch.cuda.is_available():
                self.overlap_shared = True
                self.ws_shared = e(self.ws.numel(), dt=torch.uint8)
                self.side_stream = torch.cuda.Stream(device=device)

    def route(self, x, logits_in=None, stream=None):
        g = self.gate
        B.moe_route(self.cfg, self.T, x, g["gate_w"], g.get("logit_bias"), g.get("select_bias"),
                    logits_in, self.topk_ids, self.topk_w, self.ws, stream)

    def dispatch(self, x, stream=None):
        if self.fp8_activations:      # x was quantised by forward()
            B.moe_dispatch_fp8q(self.cfg, self.T, self.xq, self.xq_scales, self.topk_ids, self.counts,
                                self.offsets, self.perm, self.inv, self.xs_q, self.xs_scales, self.ws,
                                stream)
            return
        B.moe_dispatch(self.cfg, self.T, x, self.topk_ids, self.counts, self.offsets, self.perm,
                       self.inv, self.xs, self.ws, stream)

    def expert_ffn(self, stream=None):
        w = self.experts
        if self.fp8_activations:
            B.moe_expert_ffn_fp8q(self.cfg, self.cfg.n_local, self.xs_q, self.xs_scales, self.offsets,
                                  self.T * self.cfg.top_k, w["w_gate"], w["w_up"], w["w_down"],
                                  w["s_gate"], w["s_up"], w["s_down"], self.ys, self.ws, stream)
            return
        B.moe_expert_ffn(self.cfg, self.cfg.n_local, self.xs, self.offsets, self.T * self.cfg.top_k,
                         w["w_gate"], w["w_up"], w["w_down"], w.get("s_gate"), w.get("s_up"),
                         w.get("s_down"), self.ys, self.ws, stream)

    def shared_ffn(self, x, stream=None, ws=None):
        w = self.shared
        if self.fp8_activations:      # on the rows forward() quantised
            B.moe_expert_ffn_fp8q(self.cfg, 1, self.xq, self.xq_scales, self.shared_offsets, self.T,
                                  w["w_gate"], w["w_up"], w["w_down"], w["s_gate"], w["s_up"],
                                  w["s_down"], self.shared_ys, self.ws if ws is None else ws, stream)
            return
        B.moe_expert_ffn(self.cfg, 1, x, self.shared_offsets, self.T, w["w_gate"], w["w_up"],
                         w["w_down"], w.get("s_gate"), w.get("s_up"), w.get("s_down"),
                         self.shared_ys, self.ws if ws is None else ws, stream)

    def combine(self, stream=None, ys=None):
        B.moe_combine(self.cfg, self.T, self.ys if ys is None else ys, self.inv, self.topk_w,
                      self.shared_ys, self.out, stream)

    def capture(self, x, forced=None, warmup=2):
        """Record one pass over `x` (and this object's buffers) into a HIP graph and
        return it; `graph.replay()` re-runs the pass, e.g. after new data has been
        copied into `x`.  The library clears its counters with kernels, not memset
        nodes, and opts into large LDS on a kernel's first launch, which the
        warm-up passes get out of the way before the capture starts."""
        side = torch.cuda.Stream(device=self.dev)
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for _ in range(warmup):
                self.forward(x, forced)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.forward(x, forced)
        return graph

    def forward(self, x, forced=None, stream=None):
        """One pass of the whole path.  `forced` = (ids, w) device tensors to
        bypass the gate (forced-routing stress case)."""
        concurrent = self.shared is not None and self.overlap_shared
        if self.fp8_activations:
            B.moe_quant_act(self.cfg, self.T, x, self.xq, self.xq_scales, stream)
        if concurrent:
            main = torch.cuda.current_stream() if stream is None else stream
            if isinstance(main, int):                # a raw hipStream_t handle
                main = torch.cuda.ExternalStream(main)
            self.side_stream.wait_stream(main)       # x ready; the previous combine has read shared_ys
            self.shared_ffn(x, self.side_stream, ws=self.ws_shared)
        if forced is None:
            self.route(x, stream=stream)
        else:
            self.topk_ids, self.topk_w = forced
        self.dispatch(x, stream)
        self.expert_ffn(stream)
        if concurrent:
            main.wait_stream(self.side_stream)
        elif self.shared is not None:
            self.shared_ffn(x, stream)
        self.combine(stream)
        return self.out
