#!/usr/bin/env python3
"""Benchmark of one GPU's MoE-layer share: route -> dispatch -> expert FFN ->
combine on seeded synthetic layers, one JSON line on stdout.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4|c2p|c2d|c2x|c3|c3d|c4w|c4q|c5|c1]

The default workload is c4 (the largest single-GPU configuration: the DeepSeek-R1-
shaped TP=2 x EP share at 16 384 prefill tokens); with it the line also carries a
`per_workload` table (c2p, c3, c5, c2d: shorter measurements of the same kind).

A step is one pass of the whole path over one batch, inputs resident in HBM.
`value` is tokens/s of the share; `roofline` prices the dominant kernel against
MI355X's published peaks using the kernel's algorithmic flops / bytes and its
duration measured with HIP events on the stream it runs on; `cpu_baseline` is
the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0
PEAK_MFMA_TFLOPS = {"bf16": 2500.0, "fp8": 2500.0, "f32": 157.3}   # fp8 weights run on the bf16 MFMA

DESCR = {
    "c1": "tiny fp32 layer: 64 tokens, hidden 256, 8 experts top-2, I 512",
    "c2p": "Qwen3-30B-A3B-shaped full layer, prefill 4096 tokens: hidden 2048, 128 experts top-8, I 768, bf16",
    "c2d": "Qwen3-30B-A3B-shaped full layer, decode 64 tokens: hidden 2048, 128 experts top-8, I 768, bf16",
    "c3": "Qwen3-235B-A22B-shaped EP=8 share: 8192 tokens, hidden 4096, 16 of 128 experts, I 1536, bf16",
    "c2x": "Qwen3-30B-A3B-shaped full layer, the largest prefill step (16 x 4096 tokens): hidden 2048, 128 experts top-8, I 768, bf16",
    "c3d": "Qwen3-235B-A22B-shaped EP=8 share, decode 256 tokens: hidden 4096, 16 of 128 experts, I 1536, bf16",
    "c4": "DeepSeek-R1-shaped TP=2 x EP share: 16384 tokens, hidden 7168, 32 of 256 experts + shared, I 1024, bf16",
    "c4w": "the c4 share with e4m3 block-128 weights and bf16 activations (weight tiles widened to bf16 in the tall-tile kernel)",
    "c4q": "the c4 share with e4m3 block-128 weights and expert-FFN activations quantised 1x128 to e4m3 (fp8 MFMA)",
    "c5": "DeepSeek-R1-shaped decode stress: 256 tokens, fp8-e4m3 block-128 weights, forced Zipf routing",
}


def algorithmic_work(w, a_loc, e_touched, tokens_local):
    """Per step, per kernel id: (flops, bytes) the method itself must do / move."""
    ab = 4 if w.act_dtype == "f32" else 2
    wb = {"f32": 4, "bf16": 2, "fp8": 1}[w.weight_dtype]
    T, H, E, k, I = w.T, w.H, w.E, w.k, w.I_loc
    A = T * k
    sh = T if w.shared_expert else 0
    sh_e = 1 if w.shared_expert else 0
    work = {
        "gate_gemm": (2.0 * T * H * E, T * H * ab + E * H * ab),
        "select": (0.0, T * (4 * E + 8 * k)),
        "dispatch_gather": (0.0, tokens_local * H * ab + a_loc * H * ab + A * 4),
        "dispatch_hist": (0.0, A * 4),
        "dispatch_scatter": (0.0, A * 4 + A * 4 + a_loc * 4),
        "ffn_gemm1": (4.0 * (a_loc + sh) * H * I, (e_touched + sh_e) * 2 * I * H * wb + (a_loc + sh) * H * ab),
        "ffn_gemm2": (2.0 * (a_loc + sh) * H * I, (e_touched + sh_e) * I * H * wb + (a_loc + sh) * H * ab),
        "combine": (0.0, (a_loc + sh) * H * ab + A * 8 + T * H * 4),
    }
    return work


def measure(moe, name, steps, warmup, args, full):
    """One workload: build the layer, time `steps` whole steps between two device
    synchronisations, and return the fields of the benchmark line.  `full`: also
    the HIP-graph replay, the collective-ready layouts and the CPU baseline."""
    import numpy as np
    import torch
    from workloads import gen
    from paper_2601_08800_amd.layer import config_from_workload, to_device

    w = gen.CONFIGS[name]
    t0 = time.time()
    x_np, gate = gen.make_x(w), gen.make_gate(w)
    experts = gen.make_local_experts(w)
    shared = gen.make_shared_expert(w) if w.shared_expert else None
    forced_np = gen.make_forced_routing(w) if w.zipf_s is not None else None
    print("%s: inputs generated in %.1f s" % (name, time.time() - t0), file=sys.stderr, flush=True)

    L = moe.MoELayerShare(config_from_workload(w), w.T, gate, experts, shared,
                          fp8_activations=w.fp8_activations)
    x = to_device(x_np)
    forced = None if forced_np is None else (to_device(forced_np[0]), to_device(forced_np[1]))

    if args.calibration_copy and full:
        # a copy of known size: rocprofv3 FETCH_SIZE / WRITE_SIZE of this dispatch
        # give the factor that turns the counters into bytes
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(warmup):
        L.forward(x, forced)
    torch.cuda.synchronize()
    # untimed pass with an event pair around every kernel: the per-stage table,
    # and which kernel dominates the step.  The shared expert normally runs on a
    # second stream beside the routed path; for this pass everything is put on one
    # stream so that each kernel's duration is its own.
    if args.one_stream:
        L.overlap_shared = False
    overlap = L.overlap_shared
    L.overlap_shared = False
    moe.moe_profile_enable(64 * max(steps, 1))
    for _ in range(steps):
        L.forward(x, forced)
    torch.cuda.synchronize()
    prof = moe.moe_profile_read()
    dom = max((n for n in prof if n.startswith(("ffn_gemm", "gate_gemm", "combine", "dispatch_gather"))),
              key=lambda n: prof[n][0])
    # timed region: only the dominant kernel carries events (two records per
    # launch), so the region is not slowed down by the other launches' events
    moe.moe_profile_filter([dom])
    L.overlap_shared = overlap
    for _ in range(2):
        L.forward(x, forced)
    torch.cuda.synchronize()
    moe.moe_profile_read()
    t0 = time.perf_counter()
    for _ in range(steps):
        L.forward(x, forced)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof_timed = moe.moe_profile_read()
    moe.moe_profile_filter(None)
    moe.moe_profile_enable(0)
    ms_per_step = (t1 - t0) * 1e3 / steps
    value = w.T / (ms_per_step * 1e-3)

    # spread of single steps: at least 30 steps, each between two events on the
    # stream the step starts and ends on (the side stream joins before combine)
    n_single = max(30, steps)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(n_single)]
    for a, b in evs:
        a.record()
        L.forward(x, forced)
        b.record()
    torch.cuda.synchronize()
    single = sorted(a.elapsed_time(b) for a, b in evs)
    step_stats = {"n": n_single, "median_ms": round(single[n_single // 2], 4), "min_ms": round(single[0], 4),
                  "max_ms": round(single[-1], 4)}

    counts = L.counts.cpu().numpy()
    inv = L.inv.cpu().numpy().reshape(w.T, w.k)
    a_loc = int(counts.sum())
    e_touched = int((counts > 0).sum())
    tokens_local = int((inv >= 0).any(axis=1).sum())
    n_rescored = 0
    if forced is None:          # the counter lives in the workspace: read it right after a route call
        L.route(x)
        torch.cuda.synchronize()
        n_rescored = int(L.ws[:4].view(torch.int32).item())
    work = algorithmic_work(w, a_loc, e_touched, tokens_local)

    stages = {}
    for kname, (ms, n) in prof.items():
        us = ms * 1e3 / steps
        st = {"us_per_step": round(us, 2), "launches_per_step": n / steps}
        if kname in work and us > 0:
            fl, by = work[kname]
            st["GBps"] = round(by / (us * 1e-6) / 1e9, 1)
            if fl:
                st["TFLOPs"] = round(fl / (us * 1e-6) / 1e12, 1)
        stages[kname] = st

    fl, by = work[dom]
    # measured inside the timed region; with the shared expert on a second stream
    # the kernels of the two streams share the CUs, so the one-stream pass is used
    dur = (prof[dom][0] if overlap else prof_timed[dom][0]) * 1e-3 / steps
    n_launch = (prof[dom][1] if overlap else prof_timed[dom][1]) / steps
    peak_tf = 5000.0 if w.fp8_activations else PEAK_MFMA_TFLOPS[w.weight_dtype]   # fp8 x fp8 MFMA
    t_mfma = fl / (peak_tf * 1e12)
    t_hbm = by / (PEAK_HBM_GBS * 1e9)
    if t_mfma >= t_hbm:
        roof = {"bound": "mfma", "achieved": round(fl / dur / 1e12, 2), "peak": peak_tf,
                "unit": "TFLOP/s"}
    else:
        roof = {"bound": "hbm", "achieved": round(by / dur / 1e9, 1), "peak": PEAK_HBM_GBS,
                "unit": "GB/s"}
    roof["frac"] = round(roof["achieved"] / roof["peak"], 4)
    roof["traffic"] = None
    roof["kernel"] = dom
    roof["kernel_us"] = round(dur * 1e6, 2)
    roof["launches_per_step"] = n_launch
    roof["duration_from"] = "one-stream pass (the timed step overlaps the shared expert on a second stream)" \
        if overlap else "timed region"
    roof["algorithmic_flops"] = fl
    roof["algorithmic_bytes"] = by
    roof["other_bound_frac"] = round((t_hbm if t_mfma >= t_hbm else t_mfma) / dur, 4)
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        try:
            roof["traffic"] = json.load(open(tpath)).get(name, {}).get(dom)
        except Exception:
            pass

    out = {
        "metric": "moe_layer_share_tokens_per_s", "value": round(value, 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "fp8" if w.fp8_activations else {"f32": "f32", "bf16": "bf16", "fp8": "bf16"}[w.weight_dtype],
        "data": "synthetic",
        "config": {"workload": "%s: %s" % (w.name, DESCR[w.name]), "tokens": w.T, "hidden": w.H,
                   "experts": w.E, "top_k": w.k, "local_experts": w.E_loc,
                   "inter_local": w.I_loc, "local_assignments": a_loc,
                   "tokens_rescored_fp64": n_rescored, "shared_expert_on_second_stream": bool(overlap),
                   "weight_dtype": w.weight_dtype},
        "single_steps": step_stats,
        "roofline": roof,
        "stages": stages,
    }
    if not full:
        return out

    if not args.no_extras:
        # the same step replayed from a HIP graph (launch overhead off the critical path)
        try:
            graph = L.capture(x, forced)
            for _ in range(3):
                graph.replay()
            torch.cuda.synchronize()
            g0 = time.perf_counter()
            for _ in range(steps):
                graph.replay()
            torch.cuda.synchronize()
            g_ms = (time.perf_counter() - g0) * 1e3 / steps
            out["hip_graph_replay"] = {"ms_per_step": round(g_ms, 4), "tokens_per_s": round(w.T / (g_ms * 1e-3), 1)}
            del graph
        except Exception as exc:            # reported, never fatal for the benchmark line
            out["hip_graph_replay"] = {"error": str(exc)[:200]}
        out["next_rows"] = next_rows(moe, L, w, x, a_loc, tokens_local, max(steps, 5))
        if forced is not None:
            out["route_separately"] = route_separately(moe, L, x, max(steps, 5))
        if w.act_dtype == "bf16":
            out["library_gemm"] = library_gemm(w, a_loc, tokens_local)
    # what the matrix units of this machine sustain with nothing else going on (a
    # register-only MFMA loop, ~10 ms so that the clock settles): the power-limited
    # ceiling of any bf16 GEMM here, beside the published peak the roofline is priced at
    try:
        tf = moe.moe_probe_mfma_rate(1024, 8000)
        out["mfma_probe"] = {"TFLOPs": round(tf, 1), "frac_of_published_peak": round(tf / 2500.0, 4),
                             "kernel": "register-only v_mfma_f32_32x32x16_bf16 loop, 1024 workgroups x 8 wavefronts"}
    except Exception as exc:
        out["mfma_probe"] = {"error": str(exc)[:200]}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, x_np, gate, experts, shared, forced_np,
                                           args.cpu_seconds)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c4", choices=list(DESCR))
    ap.add_argument("--also", default=None,
                    help="comma-separated workloads for the per_workload table "
                         "(default: c2p,c3,c5,c2d with the default workload, none otherwise)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the HIP-graph replay, the next_rows measurements and the per_workload table (profiling runs)")
    ap.add_argument("--one-stream", action="store_true",
                    help="keep the shared expert on the main stream in every pass (profiling runs: each "
                         "kernel's duration is then its own)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs one GPU's share on one GPU; --gpus %d is not supported "
              "(no collectives, no sharding across GPUs)" % args.gpus, file=sys.stderr)
        return 2

    import torch
    import paper_2601_08800_amd as moe

    if not torch.cuda.is_available():
        print("bench.py: no GPU", file=sys.stderr)
        return 2
    moe.load_library()                      # fails loudly when the HIP library is not built
    out = measure(moe, args.workload, args.steps, args.warmup, args, True)
    also = args.also
    if also is None:
        also = "c2p,c3,c5,c2d" if (args.workload == "c4" and not args.no_extras) else ""
    table = {}
    for name in [n for n in also.split(",") if n]:
        torch.cuda.empty_cache()
        r = measure(moe, name, args.steps, min(args.warmup, 3), args, False)
        table[name] = {"tokens_per_s": r["value"], "ms_per_step": r["ms_per_step"],
                       "single_steps": r["single_steps"], "roofline": r["roofline"],
                       "tokens_rescored_fp64": r["config"]["tokens_rescored_fp64"],
                       "stage_us": {k: v["us_per_step"] for k, v in r["stages"].items()}}
    if table:
        out["per_workload"] = table
    print(json.dumps(out), flush=True)
    return 0


def library_gemm(w, a_loc, tokens_local):
    """Context, not part of the path and not a target: the vendor library's dense bf16
    GEMM (torch.matmul) on ONE matrix with the row count of this workload's GEMM-1 and
    GEMM-2 (routed rows + shared-expert rows as a single group), 40 launches after 40
    warm-up launches, Gaussian operands like the workload's."""
    import torch
    rows = a_loc + (w.T if w.shared_expert else 0)
    if rows < 1:
        return None
    res = {"rows": rows, "note": "torch.matmul, one dense group of all rows; the path's GEMMs are ragged groups"}
    gen_ = torch.Generator(device="cuda").manual_seed(7)
    for name, n, k in (("gemm1", 2 * w.I_loc, w.H), ("gemm2", w.H, w.I_loc)):
        try:
            a = (torch.randn(rows, k, device="cuda", generator=gen_) * 0.5).to(torch.bfloat16)
            b = (torch.randn(n, k, device="cuda", generator=gen_) * 0.02).to(torch.bfloat16)
            for _ in range(40):
                c = a @ b.t()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(40):
                c = a @ b.t()
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / 40
            res[name] = {"us": round(us, 1), "TFLOPs": round(2.0 * rows * n * k / us / 1e6, 1)}
            del a, b, c
        except Exception as exc:
            res[name] = {"error": str(exc)[:200]}
    return res


def route_separately(moe, L, x, steps):
    """Workloads with forced routing skip the gate inside the timed step; the
    route of the same layer (normal gate on the same tokens) is timed here on
    its own: kernel durations from HIP events, per call."""
    import torch
    for _ in range(3):
        L.route(x)
    torch.cuda.synchronize()
    moe.moe_profile_filter(None)
    moe.moe_profile_enable(16 * steps + 16)
    for _ in range(steps):
        L.route(x)
    torch.cuda.synchronize()
    rec = moe.moe_profile_read()
    moe.moe_profile_enable(0)
    res = {name: round(ms * 1e3 / steps, 2) for name, (ms, n) in rec.items()}
    res["us"] = round(sum(res.values()), 2)
    res["tokens_rescored_fp64"] = int(L.ws[:4].view(torch.int32).item())
    return res


def next_rows(moe, L, w, x, a_loc, tokens_local, steps):
    """The collective-ready layouts of the fused schedules, measured on their
    own (they are not part of the timed step): the hidden-column shard dispatch
    of one TP rank, and one stage of the staged combine on one column block,
    overwriting and accumulating.  Kernel durations from HIP events; GB/s on
    the algorithmic bytes of the shard / block."""
    import torch
    cfg = L.cfg
    m = w.tp if w.tp > 1 else 8                    # ranks of the intra-node TP group
    if w.H % m or (w.H // m) % 8:
        return None
    ab = 4 if w.act_dtype == "f32" else 2
    T, k, Hs = w.T, w.k, w.H // m
    A = T * k
    xs_shard = torch.empty((A, Hs), dtype=L.xs.dtype, device=L.xs.device)
    ys_block = torch.empty((max(a_loc, 1), Hs), dtype=L.ys.dtype, device=L.ys.device).normal_()
    out_block = torch.zeros((T, Hs), dtype=torch.float32, device=L.ys.device)
    res = {"tp_size": m, "shard_columns": Hs}

    def timed(fn, kernel):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        moe.moe_profile_enable(16 * steps)
        moe.moe_profile_filter([kernel])
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        ms = moe.moe_profile_read()[kernel][0]
        moe.moe_profile_filter(None)
        moe.moe_profile_enable(0)
        return ms * 1e3 / steps

    us = timed(lambda: moe.moe_dispatch_shard(cfg, T, x, L.topk_ids, 0, m, L.counts, L.offsets,
                                              L.perm, L.inv, xs_shard, L.ws), "dispatch_gather")
    by = tokens_local * Hs * ab + a_loc * Hs * ab + A * 4
    res["dispatch_shard_gather"] = {"us": round(us, 2), "GBps": round(by / us / 1e3, 1)}
    for acc, name in ((0, "combine_stage"), (1, "combine_stage_accumulate")):
        us = timed(lambda: moe.moe_combine_stage(cfg, T, ys_block, L.inv, L.topk_w, m, acc,
                                                 out_block), "combine")
        by = a_loc * Hs * ab + A * 8 + T * Hs * 4 * (2 if acc else 1)
        res[name] = {"us": round(us, 2), "GBps": round(by / us / 1e3, 1)}
    return res


def cpu_baseline(w, x_np, gate, experts, shared, forced_np, budget_s):
    """The oracle as it stands, timed on the host cores on the first n tokens of
    the same batch (route + dispatch + expert MLP + combine); n grows until the
    run takes about `budget_s` seconds."""
    import numpy as np
    import oracle

    dec = lambda d: None if d is None else {
        k: (oracle.decode(v) if (v is not None and k.startswith("w_")) else v) for k, v in d.items()}
    ex, sh = dec(experts), dec(shared)
    gw = oracle.decode(gate["gate_w"])
    xf = oracle.decode(x_np)

    def run(n):
        t0 = time.perf_counter()
        if forced_np is None:
            ids, wts, _ = oracle.route(xf[:n], gw, w.k, w.score_fn, w.renormalize, w.routed_scale,
                                       w.n_groups, w.topk_groups, w.group_score_n,
                                       gate["logit_bias"], gate["select_bias"])
        else:
            ids, wts = forced_np[0][:n], forced_np[1][:n]
        oracle.layer_share(xf[:n], ids, wts, w.expert_lo, w.e_hi, ex, sh,
                           fp8_activations=w.fp8_activations)
        return time.perf_counter() - t0

    n = min(w.T, 8)
    dt = run(n)
    while dt < budget_s / 4 and n < w.T:
        n = min(w.T, max(n + 1, int(n * min(8.0, budget_s / max(dt, 1e-3)) * 0.8)))
        dt = run(n)
    sample = "first %d of %d tokens of the same batch, %.1f s" % (n, w.T, dt)
    if n == w.T and dt < budget_s / 2:
        # the whole batch is quick: repeat it until about budget_s seconds of work are timed
        reps = min(16, int(budget_s / max(dt, 1e-3)) + 1)
        dt = sum(run(n) for _ in range(reps)) / reps
        sample = "the whole batch of %d tokens, %d times, %.1f s each" % (n, reps, dt)
    return {"value": round(n / dt, 2), "unit": "tokens/s", "cores": oracle.num_threads(),
            "kind": "oracle", "sample": sample}


if __name__ == "__main__":
    sys.exit(main())
