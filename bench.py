#!/usr/bin/env python3
"""Benchmark of the per-layer recompute-and-backward path on one MI355X.

A step is one pass of the whole hot path over one synthetic micro-batch:
lynx_layer_forward(policy) -> lynx_recompute(all missing) -> lynx_layer_backward.
The headline value is the throughput of recompute + backward (the cost the
paper's scheduler moves around); forward time is reported next to it.

Prints ONE JSON line on stdout.  Everything else goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_FP32_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0

# HBM-side bytes per launch (L2 misses + write-backs) of the dense GEMM groups, from the two
# hardware-counter runs summarised in profiles/bench_C4_full_recompute_hbm_traffic.md
# (FETCH_SIZE and WRITE_SIZE, scaled by a plain copy of known size).  Not measured live:
# counters need the profiler around the process.
MEASURED_TRAFFIC_BYTES = {("C4", "full"): {
    "b12_fc2_dgrad_wgrad": 2297.5e6, "b10_fc1_dgrad_wgrad": 2131.0e6, "b2_qkv_dgrad_wgrad": 2101.5e6,
    "b7_proj_dgrad_wgrad": 1240.0e6, "op10_fc1_gemm": 809.0e6, "op12_fc2_gemm": 1009.7e6,
    "op2_qkv_gemm": 664.8e6, "op7_attn_proj_gemm": 545.2e6}}

POLICIES = {"store_all": 0x3FFF, "full": 0x2001, "attention_only": 0x3FFF & ~0x0038,
            "elementwise_only": 0x3FFF & ~0x0830}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def slot_work(cfg):
    """Algorithmic work per kernel group: slot name -> ("mfma"|"hbm", flops or bytes)."""
    e = 2 if cfg.dtype == 1 else 4
    T, h, p, f, s = cfg.tokens, cfg.hidden, cfg.proj, cfg.local_ffn, cfg.seq
    tri = cfg.micro_batch * cfg.local_heads * s * (s + 1) // 2
    d = cfg.head_dim
    lin = lambda n, k: 2.0 * T * n * k
    att = 2.0 * tri * d
    return {
        "op1_layernorm1": ("hbm", 2 * T * h * e), "op2_qkv_gemm": ("mfma", lin(3 * p, h)),
        "op3_scores": ("mfma", att), "op4_softmax_dropout": ("hbm", 3 * tri * e),
        "op5_attn_dropout": ("hbm", 2 * tri * e), "op6_context": ("mfma", att),
        "op7_attn_proj_gemm": ("mfma", lin(h, p)), "op8_bias_dropout_add1": ("hbm", 3 * T * h * e),
        "op9_layernorm2": ("hbm", 2 * T * h * e), "op10_fc1_gemm": ("mfma", lin(f, h)),
        "op11_gelu": ("hbm", 2 * T * f * e), "op12_fc2_gemm": ("mfma", lin(h, f)),
        "op13_bias_dropout_add2": ("hbm", 3 * T * h * e),
        "b13_dropout_bwd": ("hbm", 2 * T * h * e), "b12_fc2_dgrad_wgrad": ("mfma", 2 * lin(h, f)),
        "b11_gelu_bwd": ("hbm", 3 * T * f * e), "b10_fc1_dgrad_wgrad": ("mfma", 2 * lin(f, h)),
        "b98_layernorm2_dropout_bwd": ("hbm", 5 * T * h * e),
        "b7_proj_dgrad_wgrad": ("mfma", 2 * lin(h, p)),
        "b6_dpd": ("mfma", att), "b6_dv": ("mfma", att), "b54_softmax_dropout_bwd": ("hbm", 3 * tri * e),
        "b3_dq": ("mfma", att), "b3_dk": ("mfma", att), "b2_qkv_dgrad_wgrad": ("mfma", 2 * lin(3 * p, h)),
        "b2_bias_grad": ("hbm", T * 3 * p * e),
        "b1_layernorm1_bwd": ("hbm", 4 * T * h * e),
        # dPd = dC V^T with the dropout + softmax backward in its store pass: reads P, writes dS
        "b6_rowdot": ("hbm", 2 * T * p * e), "b654_dscores": ("hbm", 2 * tri * e),
        # attention without S, P, Pd (policies that keep none of them).  Forward: scores and
        # context, the two products an unfused run performs (the kernel forms the scores three
        # times; only the algorithmic two count).  Backward: dPd and dV likewise.
        "op3456_attention_fused": ("mfma", 2 * att), "b654_dscores_fused": ("mfma", att),
        "b6_dv_fused": ("mfma", att),
    }


def regenerated_ops(cfg, retain_mask):
    """The operators the library regenerates after a forward under retain_mask: asked of the
    library itself, on a handle in dry-run mode (bookkeeping only, nothing is launched and the
    placeholder addresses are never dereferenced)."""
    from paper_2406_08756_amd import binding as B
    fake = 256
    h = B.lynx_layer_create(cfg, fake, 1 << 60)
    B.lynx_layer_set_dry_run(h, True)
    B.lynx_layer_set_params(h, {k: fake for k in B.PARAM_FIELDS})
    B.lynx_layer_forward(h, fake, fake, retain_mask, 0)
    m = B.lynx_layer_missing_mask(h)
    B.lynx_layer_destroy(h)
    return [i for i in range(1, 14) if (m >> i) & 1]


def phase_flops(cfg, retain_mask):
    """Algorithmic matrix-product FLOPs of forward, of the regeneration the
    policy needs, and of backward."""
    w = slot_work(cfg)
    op_slot = {2: "op2_qkv_gemm", 3: "op3_scores", 6: "op6_context", 7: "op7_attn_proj_gemm",
               10: "op10_fc1_gemm", 12: "op12_fc2_gemm"}
    fwd = sum(w[n][1] for n in op_slot.values())
    ops = regenerated_ops(cfg, retain_mask)
    if 6 in ops and 5 not in ops and not (retain_mask >> 5) & 1:
        ops = ops + [3]    # operator 6 ran fused with operators 3-5: the score product is part of what it regenerates
    rec = sum(w[op_slot[i]][1] for i in ops if i in op_slot)
    bwd = sum(v for n, (kind, v) in w.items() if n.startswith("b") and kind == "mfma" and not n.endswith("_fused"))
    return fwd, rec, bwd


def cold_measure(B, torch, cfg, params, x, out, stream, reps=7):
    """The HBM-bound forward operators timed alone on cold caches: forward under a mask that
    keeps everything but the operator's output, a 1 GiB read sweep (more than the L2s and the
    256 MB memory-side cache hold, and it leaves no dirty lines), then lynx_recompute of that
    one operator between two events.  (The backward kernels have no entry point of their own;
    their in-situ figures stand alone.)"""
    full = POLICIES["store_all"]
    ws_bytes = B.lynx_workspace_bytes(cfg, full)
    ws = torch.empty(ws_bytes + 256, dtype=torch.uint8, device="cuda")
    layer = B.lynx_layer_create(cfg, (ws.data_ptr() + 255) // 256 * 256, ws_bytes)
    B.lynx_layer_set_params(layer, params)
    sweep = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")
    work = slot_work(cfg)
    ops = {"op1_layernorm1": (1 << 1), "op4_softmax_dropout": (1 << 4) | (1 << 5),
           "op8_bias_dropout_add1": (1 << 8), "op9_layernorm2": (1 << 9), "op11_gelu": (1 << 11)}
    res = {}
    for name, seg in ops.items():
        times = []
        for k in range(reps):
            B.lynx_layer_forward(layer, x, out, full & ~seg, k, stream)
            sweep.sum()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            B.lynx_recompute(layer, seg, stream)
            e1.record()
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1))
            B.lynx_layer_reset(layer)
        ms = sorted(times)[len(times) // 2]
        gbs = work[name][1] / (ms * 1e-3) / 1e9
        res[name] = {"ms": round(ms, 4), "achieved": round(gbs, 1), "unit": "GB/s", "frac": round(gbs / PEAK_HBM_GBS, 4)}
        log("cold %-24s %8.4f ms %8.1f GB/s" % (name, ms, gbs))
    B.lynx_layer_destroy(layer)
    return res


def cpu_baseline(cfg, retain_name):
    """The fp64 oracle as it stands, timed on the host cores on a bounded
    sample: as many micro-batch elements as fit in roughly 20 s (its cost is
    linear in the micro-batch size; one element is timed first to decide)."""
    import numpy as np
    import lynx_synth as synth
    from oracle import lynx_oracle as orc
    def timed(nb):
        small = cfg.with_(micro_batch=nb)
        params = synth.make_params(small)
        X, dOUT = synth.make_x(small), synth.make_dout(small)
        t0 = time.perf_counter()
        acts = orc.layer_forward(small, params, X)
        t1 = time.perf_counter()
        orc.layer_backward(small, params, acts, dOUT)
        t2 = time.perf_counter()
        return small, t0, t1, t2

    small, t0, t1, t2 = timed(1)
    nb = max(1, min(cfg.micro_batch, int(20.0 / max(t2 - t0, 1e-3))))
    if nb > 1:
        small, t0, t1, t2 = timed(nb)
    fwd, rec, bwd = phase_flops(small, POLICIES[retain_name])
    # the oracle has no policy machinery: regeneration costs what those forward
    # operators cost, so scale the measured forward by the share regenerated
    sec = (t1 - t0) * (rec / fwd) + (t2 - t1)
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": (rec + bwd) / sec / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": "micro_batch %d of %d; fp64 numpy oracle forward %.1f s + backward %.1f s; "
                      "regeneration priced as its share of forward FLOPs" % (
                          small.micro_batch, cfg.micro_batch, t1 - t0, t2 - t1)}


def overlap_measure(B, torch, layer, x, out, mask, segments, dout, dx, grads, main, workgroups, reps):
    """The paper hides regeneration behind tensor-parallel communication (phases 1-4).  On one
    GPU: the regeneration segments run on a side stream while a stand-in for the all-reduce
    (a copy of one [T, h] tensor by a fixed number of workgroups) runs on the main stream.
    Three timings per repetition, each after a fresh forward: stand-in alone, regeneration
    alone, both at once (from a common start to the later of the two ends)."""
    side = torch.cuda.Stream()          # default priority
    src, dst = torch.empty_like(x), torch.empty_like(x)
    nbytes = x.numel() * x.element_size()
    ev = lambda: torch.cuda.Event(enable_timing=True)
    t_comm = t_rec = t_both = 0.0

    def fresh_forward(k):
        B.lynx_layer_forward(layer, x, out, mask, k, main)

    def finish():
        B.lynx_layer_backward(layer, dout, dx, grads, main)

    for k in range(reps + 2):
        # stand-in alone
        fresh_forward(k)
        a, b = ev(), ev()
        a.record(main)
        B.lynx_comm_standin(dst, src, nbytes, workgroups, main)
        b.record(main)
        # regeneration alone (on the side stream, as it would run)
        c, d = ev(), ev()
        c.record(main)
        side.wait_event(c)
        c2 = ev(); c2.record(side)
        for seg in segments:
            B.lynx_recompute(layer, seg, side)
        d.record(side)
        main.wait_event(d)
        finish()
        # both at once
        fresh_forward(k)
        e, f, g = ev(), ev(), ev()
        e.record(main)
        side.wait_event(e)
        B.lynx_comm_standin(dst, src, nbytes, workgroups, main)
        for seg in segments:
            B.lynx_recompute(layer, seg, side)
        f.record(side)
        main.wait_event(f)
        g.record(main)
        finish()
        torch.cuda.synchronize()
        if k >= 2:
            t_comm += a.elapsed_time(b) / reps
            t_rec += c2.elapsed_time(d) / reps
            t_both += e.elapsed_time(g) / reps
    hidden = t_comm + t_rec - t_both
    return {"standin_bytes": nbytes, "standin_workgroups": workgroups, "standin_alone_ms": round(t_comm, 4),
            "standin_alone_gbs": round(2 * nbytes / (t_comm * 1e-3) / 1e9, 1),
            "regeneration_alone_ms": round(t_rec, 4), "concurrent_ms": round(t_both, 4),
            "hidden_ms": round(hidden, 4), "hidden_frac_of_shorter": round(hidden / max(min(t_comm, t_rec), 1e-9), 3),
            "segments": ["0x%x" % (m & 0xFFFFFFFF) for m in segments]}


def slice_bench(args):
    """The six-layer pipeline-stage slice (C5): six handles, forward 0 -> 5 under the seeded
    per-layer masks, then the reverse sweep 5 -> 0 (regeneration + backward per layer), which
    is what is timed.  Layer l's output buffer is layer l + 1's input."""
    import torch
    import lynx_synth as synth
    from paper_2406_08756_amd import binding as B
    base = synth.CONFIGS["C5"]
    L, masks = synth.C5_LAYERS, synth.c5_retain_masks()
    dev = lambda a: torch.from_numpy(a).to(torch.bfloat16).cuda()
    stream = torch.cuda.current_stream()
    layers, keep = [], []
    x0, dout = dev(synth.make_x(base)), dev(synth.make_dout(base))
    outs = [torch.empty_like(x0) for _ in range(L)]
    dxs = [torch.empty_like(x0) for _ in range(L)]
    for l in range(L):
        cfg = base.with_(layer_id=l)
        params = {k: dev(v) for k, v in synth.make_params(cfg).items()}
        grads = {k: torch.empty_like(v) for k, v in params.items()}
        nbytes = B.lynx_workspace_bytes(cfg, masks[l])
        ws = torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda")
        h = B.lynx_layer_create(cfg, (ws.data_ptr() + 255) // 256 * 256, nbytes)
        B.lynx_layer_set_params(h, params)
        layers.append(h)
        keep.append((params, grads, ws, cfg))

    def sweep(ev=None, k=0):
        if ev: ev[0].record(stream)
        for l in range(L):
            B.lynx_layer_forward(layers[l], x0 if l == 0 else outs[l - 1], outs[l], masks[l], k, stream)
        if ev: ev[1].record(stream)
        for l in reversed(range(L)):
            B.lynx_recompute(layers[l], B.LYNX_SEG_ALL_MISSING, stream)
            B.lynx_layer_backward(layers[l], dout if l == L - 1 else dxs[l + 1], dxs[l], keep[l][1], stream)
            if ev: ev[2 + (L - 1 - l)].record(stream)

    for k in range(args.warmup):
        sweep(None, k)
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(2 + L)] for _ in range(args.steps)]
    for k in range(args.steps):
        sweep(events[k], k)
    torch.cuda.synchronize()
    fwd_ms = sum(e[0].elapsed_time(e[1]) for e in events) / args.steps
    per_layer = [sum(e[1 + j].elapsed_time(e[2 + j]) for e in events) / args.steps for j in range(L)]  # layer 5 first
    total = sum(per_layer)
    flops = 0.0
    for l in range(L):
        POLICIES["m%d" % l] = masks[l]
        _, rec_f, bwd_f = phase_flops(keep[l][3], masks[l])
        flops += rec_f + bwd_f
    for h in layers:
        B.lynx_layer_destroy(h)
    print(json.dumps({
        "metric": "recompute+backward TFLOP/s per GPT layer shard", "value": round(flops / (total * 1e-3) / 1e12, 2),
        "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(total, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "C5 slice: 6 layers h=%d a=%d d=%d f=%d s=%d b=%d tp=%d, seeded masks %s" % (
            base.hidden, base.local_heads, base.head_dim, base.local_ffn, base.seq, base.micro_batch, base.tp_size,
            " ".join("%04x" % m for m in masks)),
            "timed_region": "reverse sweep: lynx_recompute + lynx_layer_backward for layers 5..0"},
        "forward_sweep_ms": round(fwd_ms, 4),
        "reverse_sweep_ms_per_layer": {"layer%d" % (L - 1 - j): round(v, 4) for j, v in enumerate(per_layer)}}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="C4", choices=["C1", "C2", "C3", "C4", "C5"])
    ap.add_argument("--policy", default=None, choices=list(POLICIES))
    ap.add_argument("--retain-mask", default=None,
                    help="explicit retain mask (hex), e.g. one of the six-layer slice's per-layer masks; overrides --policy")
    ap.add_argument("--heu", action="store_true",
                    help="choose the policy with lynx_policy_solve (Sec. 4.2) from operator times measured "
                         "in this run; see --budget-frac and --ctime-ms")
    ap.add_argument("--budget-frac", type=float, default=0.25,
                    help="--heu: memory budget = checkpoint + this fraction of the store-all activations")
    ap.add_argument("--ctime-ms", default="0.27,0.27,0.27,0.27",
                    help="--heu: the four communication windows CTime_1..4 in ms (modelled, one GPU)")
    ap.add_argument("--overlap", action="store_true",
                    help="also measure regeneration on a side stream under a stand-in for the "
                         "tensor-parallel all-reduce (lynx_comm_standin); adds an 'overlap' object")
    ap.add_argument("--standin-workgroups", type=int, default=32)
    ap.add_argument("--slice", action="store_true",
                    help="time the six-layer pipeline-stage slice (C5) instead of one layer")
    ap.add_argument("--cold", action="store_true",
                    help="also time the HBM-bound forward operators one by one after a 1 GiB read sweep "
                         "(cold caches) next to their in-situ figures")
    ap.add_argument("--zeros", action="store_true",
                    help="diagnostic: all-zero inputs and parameters (shows how far the dense products are "
                         "held back by power rather than by their schedule); the line says data=zeros")
    ap.add_argument("--fused-attention", action="store_true",
                    help="set LYNX_FLAG_FUSED_ATTENTION: no seq x seq activation under policies that drop S, P, Pd")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch one plain 1 GiB device copy (the known-size kernel that "
                         "hardware-counter runs of this command are scaled by)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")
        sys.exit(2)

    import torch
    import lynx_synth as synth
    from paper_2406_08756_amd import binding as B

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(1)
    if args.slice:
        return slice_bench(args)
    cfg = synth.CONFIGS[args.config]
    if args.fused_attention:
        cfg = cfg.with_(flags=1)
    policy = args.policy or {"C3": "elementwise_only", "C2": "full"}.get(args.config, "full")
    mask = POLICIES[policy]
    if args.retain_mask is not None:
        mask = (int(args.retain_mask, 16) & 0x3FFF) | 1
        policy = "mask_0x%04x" % mask
        POLICIES[policy] = mask
    tdtype = torch.bfloat16 if cfg.dtype == synth.BF16 else torch.float32

    def dev(a):
        t = torch.from_numpy(a)
        return (t.to(tdtype) if cfg.dtype == synth.BF16 else t).cuda()

    log("bench: config %s policy %s; generating inputs" % (args.config, policy))
    params = {k: dev(v) for k, v in synth.make_params(cfg).items()}
    x, dout = dev(synth.make_x(cfg)), dev(synth.make_dout(cfg))
    if args.zeros:
        # a diagnostic, not a benchmark line: the same launches on all-zero operands.  Nothing
        # toggles in the matrix pipes, the clock stays up, and what the dense products then
        # reach is the limit of their schedule rather than of the chip's power budget
        for t in list(params.values()) + [x, dout]:
            t.zero_()
    out, dx = torch.empty_like(x), torch.empty_like(x)
    grads = {k: torch.empty_like(v) for k, v in params.items()}
    ws_bytes = B.lynx_workspace_bytes(cfg, mask)
    ws = torch.empty(ws_bytes + 256, dtype=torch.uint8, device="cuda")
    layer = B.lynx_layer_create(cfg, (ws.data_ptr() + 255) // 256 * 256, ws_bytes)
    B.lynx_layer_set_params(layer, params)
    stream = torch.cuda.current_stream()

    segments = [B.LYNX_SEG_ALL_MISSING]
    heu = None
    if args.heu:
        # C_i: each forward operator's time under store-all, from the library's event pairs
        full_ws = torch.empty(B.lynx_workspace_bytes(cfg, POLICIES["store_all"]) + 256, dtype=torch.uint8, device="cuda")
        prof = B.lynx_layer_create(cfg, (full_ws.data_ptr() + 255) // 256 * 256, full_ws.numel() - 256)
        B.lynx_layer_set_params(prof, params)
        B.lynx_layer_set_profiling(prof, True)
        cost = [0.0] * 13
        reps = 5
        for k in range(reps + 2):
            B.lynx_layer_forward(prof, x, out, POLICIES["store_all"], k, stream)
            ms = B.lynx_layer_profile_ms(prof)
            B.lynx_layer_reset(prof)
            if k >= 2:
                for name, v in ms.items():
                    if name.startswith("op"):
                        cost[int(name[2:].split("_")[0]) - 1] += v / reps
        B.lynx_layer_destroy(prof)
        del full_ws
        # the store-all forward runs OP4 and OP5 as one kernel (its time is under OP4): split it evenly
        cost[3], cost[4] = 0.5 * cost[3], 0.5 * cost[3]
        # OP7+OP8 and OP12+OP13 run as one launch each where the matrix-core kernel applies (the
        # time is under the linear operator); run on its own, the bias + dropout + residual
        # operator moves 3 T h e bytes: price it at 5.5 TB/s, what the stand-alone kernel reaches
        # (and take about two thirds of that off the fused launch: it does the same work minus a
        # write and a read of the product)
        for lin in (7, 12):
            if cost[lin] == 0.0:
                cost[lin] = 3.0 * cfg.tokens * cfg.hidden * (2 if cfg.dtype == 1 else 4) / 5.5e9
                cost[lin - 1] = max(cost[lin - 1] - 0.65 * cost[lin], 0.5 * cost[lin - 1])
        M = [B.lynx_activation_bytes(cfg, i) for i in range(14)]
        budget = M[13] + args.budget_frac * sum(M[1:13])
        ctime = [float(v) for v in args.ctime_ms.split(",")]
        prob = B.lynx_policy_layer_problem(cfg, cost, ctime=ctime, m_budget=budget)
        heu = B.lynx_policy_solve(prob)
        if heu is None:
            log("bench.py: no policy fits the budget")
            sys.exit(1)
        mask = heu["retain_mask"]
        policy = "heu_0x%04x" % mask
        POLICIES[policy] = mask
        # phases 1-4 are what the communication windows would hide; phase 5 is left to backward
        segments = [m for m in heu["phase_mask"][:4] if m]
        heu = dict(heu, cost_ms=[round(c, 4) for c in cost], ctime_ms=ctime, budget_bytes=budget,
                   phase_ops=[[i for i in range(1, 14) if (m >> i) & 1] for m in heu["phase_mask"]])
        log("bench: HEU policy retain 0x%04x phases %s critical %.3f ms of %.3f ms regenerated" % (
            mask, heu["phase_ops"], heu["critical_cost"], heu["recompute_cost"]))
        ws_bytes = B.lynx_workspace_bytes_for_schedule(cfg, mask, heu["phase_mask"][:4])
        B.lynx_layer_destroy(layer)
        ws = torch.empty(ws_bytes + 256, dtype=torch.uint8, device="cuda")
        layer = B.lynx_layer_create(cfg, (ws.data_ptr() + 255) // 256 * 256, ws_bytes)
        B.lynx_layer_set_params(layer, params)

    def step(ev=None, k=0):
        if ev: ev[0].record(stream)
        B.lynx_layer_forward(layer, x, out, mask, k, stream)
        if ev: ev[1].record(stream)
        for seg in segments:
            B.lynx_recompute(layer, seg, stream)
        if ev: ev[2].record(stream)
        B.lynx_layer_backward(layer, dout, dx, grads, stream)
        if ev: ev[3].record(stream)

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        torch.empty_like(src).copy_(src)
        del src
    for k in range(args.warmup):
        step(None, k)
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(events[k], k)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    fwd_ms = sum(e[0].elapsed_time(e[1]) for e in events) / args.steps
    rec_ms = sum(e[1].elapsed_time(e[2]) for e in events) / args.steps
    bwd_ms = sum(e[2].elapsed_time(e[3]) for e in events) / args.steps
    per_step = sorted(e[1].elapsed_time(e[3]) for e in events)
    median_ms, min_ms = per_step[len(per_step) // 2], per_step[0]

    # per-kernel durations: the same steps again with the library's event pairs on
    B.lynx_layer_set_profiling(layer, True)
    acc, cnt = {}, {}
    def collect(prefix):
        for name, ms in B.lynx_layer_profile_ms(layer).items():
            key = prefix + name if name.startswith("op") else name
            acc[key] = acc.get(key, 0.0) + ms
            cnt[key] = cnt.get(key, 0) + 1

    for k in range(args.steps):
        B.lynx_layer_forward(layer, x, out, mask, k, stream)
        collect("fwd/")
        for seg in segments:
            B.lynx_recompute(layer, seg, stream)
        B.lynx_layer_backward(layer, dout, dx, grads, stream)
        collect("rec/")
    B.lynx_layer_set_profiling(layer, False)
    overlap = None
    if args.overlap:
        overlap = overlap_measure(B, torch, layer, x, out, mask, segments, dout, dx, grads, stream,
                                  args.standin_workgroups, max(args.steps, 5))
    B.lynx_layer_destroy(layer)
    cold = cold_measure(B, torch, cfg, params, x, out, stream) if args.cold else None

    # What a plain device copy of one [T, h] tensor reaches on this machine, cold (four buffer
    # pairs in rotation, 1.3 GB: past the 256 MB memory-side cache): the practical ceiling
    # for the HBM-bound kernels, quoted beside each of them.
    n_copy = cfg.tokens * cfg.hidden
    pairs = [(torch.zeros(n_copy, dtype=tdtype, device="cuda"), torch.empty(n_copy, dtype=tdtype, device="cuda"))
             for _ in range(4)]
    for a, b in pairs:
        b.copy_(a)
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record(stream)
    for rep in range(3):
        for a, b in pairs:
            b.copy_(a)
    c1.record(stream)
    torch.cuda.synchronize()
    copy_gbs = 12 * 2 * n_copy * x.element_size() / (c0.elapsed_time(c1) * 1e-3) / 1e9
    del pairs

    work = slot_work(cfg)
    mfma_peak = PEAK_BF16_TFLOPS if cfg.dtype == synth.BF16 else PEAK_FP32_TFLOPS
    kernels = {}
    for name in acc:
        ms = acc[name] / cnt[name]
        kind, amount = work[name.split("/")[-1]]
        if name == "fwd/op4_softmax_dropout" and not (mask >> 4) & 1:
            amount = amount * 2 // 3      # forward under this policy does not store P
        if kind == "mfma":
            ach = amount / (ms * 1e-3) / 1e12
            kernels[name] = {"ms": round(ms, 4), "bound": "mfma", "achieved": round(ach, 2),
                             "unit": "TFLOP/s", "frac": round(ach / mfma_peak, 4)}
            # the attention products move one seq x seq tensor (the causal triangle) for a contraction
            # of only head_dim: they sit on the HBM side of the ridge, so quote them against it too
            if name.split("/")[-1] in ("op3_scores", "op6_context", "b6_dpd", "b6_dv", "b3_dq", "b3_dk"):
                tri_bytes = cfg.micro_batch * cfg.local_heads * cfg.seq * (cfg.seq + 1) // 2 * x.element_size()
                gbs = tri_bytes / (ms * 1e-3) / 1e9
                kernels[name].update({"hbm_achieved": round(gbs, 1), "hbm_unit": "GB/s of the causal triangle",
                                      "hbm_frac": round(gbs / PEAK_HBM_GBS, 4),
                                      "frac_of_copy": round(gbs / copy_gbs, 4)})
        else:
            ach = amount / (ms * 1e-3) / 1e9
            kernels[name] = {"ms": round(ms, 4), "bound": "hbm", "achieved": round(ach, 1),
                             "unit": "GB/s", "frac": round(ach / PEAK_HBM_GBS, 4),
                             "frac_of_copy": round(ach / copy_gbs, 4)}
    log("plain cold copy of one [T, h] tensor: %.1f GB/s (%.3f of 8 TB/s)" % (copy_gbs, copy_gbs / PEAK_HBM_GBS))
    log("%-28s %9s %6s %10s %8s %8s" % ("kernel group", "ms", "bound", "achieved", "frac", "of copy"))
    for name, k in kernels.items():
        log("%-28s %9.4f %6s %10.1f %8.3f %8s" % (name, k["ms"], k["bound"], k["achieved"], k["frac"],
                                                   "%.3f" % k["frac_of_copy"] if "frac_of_copy" in k else ""))

    # dominant kernel: the dense linear-layer products (forward, dgrad, wgrad share
    # one kernel family); quote the one with the most time per step
    dense = [n for n in kernels if kernels[n]["bound"] == "mfma"
             and ("gemm" in n or n.endswith("dgrad_wgrad"))]
    dom = max(dense, key=lambda n: kernels[n]["ms"])
    traffic = MEASURED_TRAFFIC_BYTES.get((args.config, policy), {}).get(dom.split("/")[-1])
    roofline = {"bound": "mfma", "kernel": dom, "achieved": kernels[dom]["achieved"], "peak": mfma_peak,
                "unit": "TFLOP/s", "frac": kernels[dom]["frac"], "traffic": traffic,
                "traffic_unit": "bytes per launch (counter runs under profiles/, not live)",
                "ms_per_launch": kernels[dom]["ms"]}
    fused = {"b12_fc2_dgrad_wgrad": "the launch also applies the GeLU backward and sums the FC1 bias gradient in its "
                                    "store pass (reads U, T*f*e bytes more); achieved counts the matrix flops only",
             "op7_attn_proj_gemm": "the launch also applies bias + dropout + residual in its store pass",
             "op12_fc2_gemm": "the launch also applies bias + dropout + residual in its store pass"}
    if dom.split("/")[-1] in fused and cfg.dtype == synth.BF16:
        roofline["note"] = fused[dom.split("/")[-1]]

    fwd_f, rec_f, bwd_f = phase_flops(cfg, mask)
    rb_ms = rec_ms + bwd_ms
    value = (rec_f + bwd_f) / (rb_ms * 1e-3) / 1e12
    result = {
        "metric": "recompute+backward TFLOP/s per GPT layer shard",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(rb_ms, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == synth.BF16 else "f32",
        "data": "zeros (diagnostic, not a benchmark figure)" if args.zeros else "synthetic",
        "config": {"workload": "%s: h=%d a=%d d=%d f=%d s=%d b=%d tp=%d, policy=%s" % (
            args.config, cfg.hidden, cfg.local_heads, cfg.head_dim, cfg.local_ffn, cfg.seq,
            cfg.micro_batch, cfg.tp_size, policy + (", fused attention" if cfg.flags & 1 else "")),
            "timed_region": "lynx_recompute(all missing) + lynx_layer_backward per step, HIP events; "
                            "each step also runs lynx_layer_forward first (forward_ms, inside wall_ms_per_step)"},
        "recompute_ms": round(rec_ms, 4), "backward_ms": round(bwd_ms, 4), "forward_ms": round(fwd_ms, 4),
        "wall_ms_per_step": round(wall_ms, 4),
        "median_ms_per_step": round(median_ms, 4), "min_ms_per_step": round(min_ms, 4),
        "algorithmic_tflop": {"forward": fwd_f / 1e12, "recompute": rec_f / 1e12, "backward": bwd_f / 1e12},
        "workspace_bytes": ws_bytes,
        "roofline": roofline,
        "hbm_copy_ceiling": {"value": round(copy_gbs, 1), "unit": "GB/s", "frac": round(copy_gbs / PEAK_HBM_GBS, 4),
                             "what": "torch copy_ of one [T, h] tensor, four buffer pairs in rotation (cold), "
                                     "read + written bytes"},
        "kernels": kernels,
    }
    if overlap is not None:
        result["overlap"] = overlap
    if cold is not None:
        result["cold_cache"] = cold
    if heu is not None:
        # recompute_ms here is what phases 1-4 regenerate (hidden behind communication in the
        # paper's schedule); backward_ms includes phase 5, the part left on the critical path
        result["heu"] = heu
    if not args.no_cpu_baseline:
        log("bench: timing the CPU oracle on a bounded sample")
        result["cpu_baseline"] = cpu_baseline(cfg, policy)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
