#!/usr/bin/env python3
"""Benchmark of the ETR MoE-layer forward on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config cfg5] [--capacity C]
                    [--no-others] [--no-cpu-baseline]

A "step" is one pass of the whole hot path (route -> select -> dispatch -> expert FFN ->
combine, one etr_moe_forward call) over one batch of seeded synthetic tokens that is
already resident in HBM.  Prints ONE JSON line.  The headline (value, roofline, cpu_baseline)
is the largest single-GPU workload, cfg5; the other bf16 workloads (cfg2, cfg3 and cfg4 at
each value of its capacity schedule) are timed after it, with fewer steps, and reported under
"other_workloads" of the same line.  Per workload: tokens/s of the whole layer, the two FFN
GEMMs against the bf16 MFMA peak (durations from HIP events recorded by the library on the
launch stream), and the HBM-bound stages called on their own against the HBM peak.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_F32_TFLOPS = 157.3       # fp32 vector
PEAK_HBM_GBS = 8000.0
INFINITY_CACHE_BYTES = 256e6  # a stage whose working set fits here is not an HBM measurement


def profiled_traffic(config: str):
    """HBM bytes per launch of the dominant kernel as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by
    what a plain copy reads on the same counters) and kept in profiles/: (bytes, file) or (None, None).  The figure
    is quoted from that file, not measured by this run."""
    path = os.path.join(ROOT, "profiles", f"moe_forward_{config}_kernels_and_traffic.txt")
    try:
        with open(path) as f:
            m = re.search(r"^# dominant_kernel_traffic_bytes_per_launch:\s*([0-9.eE+]+)", f.read(), re.M)
        return (float(m.group(1)), os.path.relpath(path, ROOT)) if m else (None, None)
    except OSError:
        return None, None


def _to_np(t):
    import numpy as np
    import torch
    t = t.detach().cpu().contiguous()
    return t.view(torch.int16).numpy().view(np.uint16) if t.dtype == torch.bfloat16 else t.numpy()


def cpu_baseline(shape, cfg, tensors, budget_tokens: int, single_thread_tokens: int):
    """Times the oracle (as it stands) on the host cores: routing on all T tokens, the expert FFN and the
    weighted sum on the first `budget_tokens` tokens, extrapolated linearly in tokens; then the same on ONE
    thread with a smaller token sample."""
    import numpy as np
    from oracle import etr_ref
    host = {k: _to_np(v) for k, v in tensors.items()}

    def leg(n):
        n = min(n, shape.T)
        t0 = time.perf_counter()
        score, _ = etr_ref.route(host["x"], host["w_emb"], shape.D, shape.dtype, cfg.cos)
        etr_ref.select(score, shape.k, cfg.capacity, cfg.mode)
        t_routing = time.perf_counter() - t0
        t0 = time.perf_counter()
        etr_ref.moe_forward(host["x"], host["w_emb"], host["w_gate"], host["w_up"], host["w_down"], D=shape.D, k=shape.k,
                            capacity=cfg.capacity, dtype=shape.dtype, mode=cfg.mode, cos_mode=cfg.cos,
                            tokens=np.arange(n, dtype=np.int32))
        t_sample = time.perf_counter() - t0
        t_full = t_routing + max(t_sample - t_routing, 0.0) * (shape.T / n)
        return shape.T / t_full, (f"routing on all {shape.T} tokens ({t_routing:.2f} s); FFN+combine on the first {n} "
                                  f"tokens ({max(t_sample - t_routing, 0.0):.2f} s), extrapolated linearly to {shape.T}")

    cores = etr_ref.num_threads()
    value, sample = leg(budget_tokens)
    etr_ref.set_num_threads(1)
    try:
        v1, s1 = leg(single_thread_tokens)
    finally:
        etr_ref.set_num_threads(cores)
    return {"value": value, "unit": "tokens/s", "cores": cores, "kind": "oracle", "sample": sample,
            "single_thread": {"value": v1, "unit": "tokens/s", "cores": 1, "sample": s1}}


def bench_backward(args, shape, cfg, t, dev):
    """K calls of etr_moe_backward on the routing of one forward call; one JSON line."""
    import torch
    from paper_2406_00023_amd import binding as B
    from paper_2406_00023_amd import inputs as I
    T, E, C, d, H = shape.T, shape.E, cfg.capacity, shape.d, shape.H
    dt = shape.torch_dtype
    score = torch.empty(T, E, dtype=torch.float32, device=dev)
    gate = torch.empty(T, E, dtype=torch.float32, device=dev)
    slot_of = torch.empty(T, E, dtype=torch.int32, device=dev)
    slot_token = torch.empty(E, C, dtype=torch.int32, device=dev)
    topk = torch.empty(T, max(shape.k, 1), dtype=torch.int32, device=dev)
    counts = torch.zeros(E, dtype=torch.int32, device=dev)
    B.etr_route(cfg, t["x"], t["w_emb"], score, gate)
    B.etr_select(cfg, score, topk, slot_of, slot_token, counts, B.alloc_workspace(B.etr_select_workspace_bytes(cfg), dev))
    dout = I.make_upstream_gradient(shape, dev)
    dx = torch.empty(T, d, dtype=dt, device=dev)
    dwg, dwu = torch.empty(E, H, d, dtype=dt, device=dev), torch.empty(E, H, d, dtype=dt, device=dev)
    dwd = torch.empty(E, d, H, dtype=dt, device=dev)
    ws = B.alloc_workspace(B.etr_backward_workspace_bytes(cfg), dev)
    a_saved = b_saved = None
    train_ms = None
    if args.saved:
        a_saved, b_saved = (torch.empty(E, C, H, dtype=dt, device=dev) for _ in range(2))
        out = torch.empty(T, d, dtype=dt, device=dev)
        wsf = B.alloc_workspace(B.etr_workspace_bytes(cfg), dev)
        fwd = lambda: B.etr_moe_forward_train(cfg, t["x"], t["w_emb"], t["w_gate"], t["w_up"], t["w_down"], out, a_saved,
                                              b_saved, wsf)
        for _ in range(args.warmup):
            fwd()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fwd()
        torch.cuda.synchronize()
        train_ms = 1e3 * (time.perf_counter() - t0) / args.steps

    def step():
        B.etr_moe_backward(cfg, t["x"], t["w_emb"], t["w_gate"], t["w_up"], t["w_down"], score, gate, slot_of,
                           slot_token, counts, dout, dx, dwg, dwu, dwd, ws, a_saved=a_saved, b_saved=b_saved)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = (time.perf_counter() - t0) / args.steps
    rows = int(counts.sum().item())
    # recompute 4dH (not with --saved) + W_d^T dout 2dH + input gradient 4dH + weight gradients 6dH per kept row
    flop = (12.0 if args.saved else 16.0) * rows * d * H
    peak = PEAK_BF16_TFLOPS if shape.dtype == I.DT_BF16 else PEAK_F32_TFLOPS
    print(json.dumps({
        "metric": "MoE-layer backward tokens/sec on 1 MI355X", "value": T / elapsed, "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": 1e3 * elapsed, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if shape.dtype == I.DT_BF16 else "f32",
        "data": "synthetic",
        "config": {"workload": f"{shape.name} backward{' (pre-activations kept by the training forward)' if args.saved else ''}: "
                               f"T={T} d={d} E={E} capacity={C} H={H}", "kept_rows": rows},
        "forward_train_ms": train_ms,
        "roofline": {"kernel": "all products of the backward pass together (grouped GEMM kernel)",
                     "bound": "mfma" if shape.dtype == I.DT_BF16 else "alu", "achieved": flop / elapsed / 1e12,
                     "peak": peak, "unit": "TFLOP/s", "frac": flop / elapsed / 1e12 / peak, "traffic": None,
                     "algorithmic_flop": flop},
    }), flush=True)


def measure_forward(shape, cfg, t, steps, warmup, dev):
    """Times `steps` fused forward calls (only the dominant kernel bracketed by events), then a second pass with
    every stage boundary marked, then the HBM-bound stages on their own.  Returns a dict of raw figures."""
    import torch
    from paper_2406_00023_amd import binding as B
    from paper_2406_00023_amd import inputs as I

    out = torch.empty(shape.T, shape.d, dtype=shape.torch_dtype, device=dev)
    counts = torch.zeros(shape.E, dtype=torch.int32, device=dev)
    ws = B.alloc_workspace(B.etr_workspace_bytes(cfg), dev)

    def step(events=None):
        if events is None:
            B.etr_moe_forward(cfg, t["x"], t["w_emb"], t["w_gate"], t["w_up"], t["w_down"], out, ws, counts=counts)
        else:
            B.etr_moe_forward_profiled(cfg, t["x"], t["w_emb"], t["w_gate"], t["w_up"], t["w_down"], out, ws, events,
                                       counts=counts)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    # timed region: K steps; only the dominant kernel (FFN gate/up GEMM) is bracketed by events
    # (boundaries 3 and 4), because every recorded event costs a few microseconds of stream time
    gemm_events = [B.StageEvents(only=(3, 4)) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(gemm_events[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    t_gemm1_ms = sum(B.elapsed_ms(ev, 3, 4) for ev in gemm_events) / steps
    # second pass, all stage boundaries marked: the per-stage breakdown (not part of `value`)
    events = [B.StageEvents() for _ in range(steps)]
    for i in range(steps):
        step(events[i])
    torch.cuda.synchronize()
    stage = [0.0] * (B.N_STAGE_EVENTS - 1)
    for ev in events:
        for i, ms in enumerate(ev.stage_ms()):
            stage[i] += ms / steps

    # the HBM-bound stages once more on their own (the fused call folds the rearrangement into GEMM-1
    # and the stage events include launch gaps): plain hipEvent timing of back-to-back stage calls
    def time_stage(fn, reps=20):
        ev = B.StageEvents()
        fn(); torch.cuda.synchronize()
        B.record_event(ev, 0)
        for _ in range(reps):
            fn()
        B.record_event(ev, 1)
        torch.cuda.synchronize()
        return B.elapsed_ms(ev, 0, 1) / reps

    E, C, T, d = shape.E, cfg.capacity, shape.T, shape.d
    score = torch.empty(T, E, dtype=torch.float32, device=dev)
    gate = torch.empty(T, E, dtype=torch.float32, device=dev)
    slot_of = torch.empty(T, E, dtype=torch.int32, device=dev)
    slot_token = torch.empty(E, C, dtype=torch.int32, device=dev)
    topk = torch.empty(T, max(shape.k, 1), dtype=torch.int32, device=dev)
    xp = torch.empty(E, C, d, dtype=shape.torch_dtype, device=dev)
    sws = B.alloc_workspace(B.etr_select_workspace_bytes(cfg), dev)
    B.etr_route(cfg, t["x"], t["w_emb"], score, gate)
    B.etr_select(cfg, score, topk, slot_of, slot_token, counts, sws)
    alone = {
        "route": time_stage(lambda: B.etr_route(cfg, t["x"], t["w_emb"], score, gate)),
        "select": time_stage(lambda: B.etr_select(cfg, score, topk, slot_of, slot_token, counts, sws)),
        "dispatch": time_stage(lambda: B.etr_dispatch(cfg, t["x"], slot_token, counts, xp)),
        "combine": time_stage(lambda: B.etr_combine(cfg, xp, gate, slot_of, out)),
    }
    rows = int(counts.sum().item())
    elt = 4 if shape.dtype == I.DT_F32 else 2
    TE = T * E
    bytes_alg = {
        "route": T * d * elt + 2 * TE * 4,
        "dispatch": rows * (2 * d * elt + 4),
        "combine": rows * d * elt + T * d * elt + TE * 8,
    }
    hbm = {}
    for k, v in bytes_alg.items():
        gbs = v / (alone[k] * 1e-3) / 1e9
        hbm[k] = {"us": round(alone[k] * 1e3, 2), "algorithmic_MB": round(v / 1e6, 1), "GBs": round(gbs, 1)}
        if v > INFINITY_CACHE_BYTES:
            hbm[k]["frac_of_8TBs"] = round(gbs / PEAK_HBM_GBS, 3)
        else:   # back-to-back calls on a working set that stays in the 256 MB Infinity Cache: not an HBM figure
            hbm[k]["frac_of_8TBs"] = None
            hbm[k]["note"] = "working set fits the Infinity Cache; latency-bound, no HBM fraction quoted"
    hbm["select"] = {"us": round(alone["select"] * 1e3, 2)}
    peak = PEAK_BF16_TFLOPS if shape.dtype == I.DT_BF16 else PEAK_F32_TFLOPS
    flops_gemm1 = 4.0 * rows * d * shape.H
    flops_gemm2 = 2.0 * rows * d * shape.H
    gemm1 = flops_gemm1 / (t_gemm1_ms * 1e-3) / 1e12
    gemm2 = flops_gemm2 / (stage[4] * 1e-3) / 1e12 if stage[4] > 0 else None
    del ws, xp
    return dict(ms_per_step=1e3 * elapsed / steps, tokens_per_s=T / (elapsed / steps), rows=rows, peak=peak,
                flops_gemm1=flops_gemm1, gemm1_TFLOPs=gemm1, gemm2_TFLOPs=gemm2,
                stage_ms={name: round(ms, 5) for name, ms in zip(B.STAGE_NAMES, stage)}, stage_alone=hbm,
                algorithmic_bytes_gemm1=elt * (2.0 * E * shape.H * d + rows * d + rows * shape.H))


def workload_name(shape, cfg):
    return (f"{shape.name}: T={shape.T} d={shape.d} E={shape.E} D={shape.D} k={shape.k} capacity={cfg.capacity} "
            f"H={shape.H} mode={('TCR', 'ECR', 'BIDIR', 'TCR_RANK', 'BIDIR_STRICT')[cfg.mode]} tokens={shape.recipe}")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="cfg5", help="headline workload (default: the largest single-GPU one)")
    ap.add_argument("--capacity", type=int, default=None, help="override the capacity (cfg4's schedule)")
    ap.add_argument("--no-others", action="store_true", help="time the headline workload only")
    ap.add_argument("--other-steps", type=int, default=20, help="timed steps of each of the other workloads")
    ap.add_argument("--cpu-tokens", type=int, default=4096, help="tokens of the oracle's FFN sample (all host cores)")
    ap.add_argument("--cpu-tokens-1", type=int, default=256, help="tokens of the oracle's FFN sample on one thread")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--backward", action="store_true",
                    help="time etr_moe_backward instead of the forward (not the headline metric; no cpu_baseline)")
    ap.add_argument("--saved", action="store_true",
                    help="with --backward: hand over the pre-activations kept by etr_moe_forward_train (no recomputation)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference for scaling rocprofv3's FETCH_SIZE/WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no collectives, no sharding); --gpus must be 1")

    import torch
    from paper_2406_00023_amd import binding as B
    from paper_2406_00023_amd import inputs as I

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    B.load_library()
    shape = I.CONFIGS[args.config]
    cfg = B.make_config(shape, capacity=args.capacity)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    t = I.make_inputs(shape, dev)
    if args.backward:
        return bench_backward(args, shape, cfg, t, dev)

    m = measure_forward(shape, cfg, t, args.steps, args.warmup, dev)
    bf16 = shape.dtype == I.DT_BF16
    traffic, traffic_file = profiled_traffic(args.config) if args.capacity is None else (None, None)
    res = {
        "metric": "MoE-layer tokens/sec on 1 MI355X",
        "value": m["tokens_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": m["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32",
        "data": "synthetic",
        "config": {"workload": workload_name(shape, cfg), "kept_rows": m["rows"]},
        "roofline": {"kernel": "gemm_bf16_persistent_kernel<GLU> (FFN gate/up projections + SwiGLU)" if bf16
                     else "gemm_f32_kernel<GLU>",
                     "bound": "mfma" if bf16 else "alu",
                     "achieved": m["gemm1_TFLOPs"], "peak": m["peak"], "unit": "TFLOP/s",
                     "frac": m["gemm1_TFLOPs"] / m["peak"],
                     "traffic": traffic,
                     "traffic_source": (f"quoted from {traffic_file} (rocprofv3 FETCH_SIZE x2.0 + WRITE_SIZE x1.0 per launch), "
                                        "not measured by this run") if traffic_file else None,
                     "algorithmic_flop": m["flops_gemm1"],
                     "algorithmic_bytes": m["algorithmic_bytes_gemm1"]},
        "stage_ms": m["stage_ms"],
        "stage_alone": m["stage_alone"],
        "ffn_down_TFLOPs": m["gemm2_TFLOPs"],
        "ffn_down_frac": m["gemm2_TFLOPs"] / m["peak"] if m["gemm2_TFLOPs"] else None,
    }
    if args.calibrate_copy:
        a = torch.ones(1 << 30, dtype=torch.uint8, device=dev)
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(shape, cfg, t, args.cpu_tokens, args.cpu_tokens_1)
    if not args.no_others and args.capacity is None:
        others = []
        del t
        torch.cuda.empty_cache()
        for name in ("cfg2", "cfg3", "cfg4", "cfg5"):
            if name == args.config:
                continue
            sh = I.CONFIGS[name]
            tt = I.make_inputs(sh, dev)
            for cap in (sh.capacity_sweep or (None,)):
                c = B.make_config(sh, capacity=cap)
                mm = measure_forward(sh, c, tt, args.other_steps, 5, dev)
                others.append({
                    "workload": workload_name(sh, c), "kept_rows": mm["rows"], "steps": args.other_steps,
                    "ms_per_step": round(mm["ms_per_step"], 4), "tokens_per_s": round(mm["tokens_per_s"], 1),
                    "ffn_gate_up_TFLOPs": round(mm["gemm1_TFLOPs"], 1),
                    "ffn_gate_up_frac": round(mm["gemm1_TFLOPs"] / mm["peak"], 4),
                    "ffn_down_TFLOPs": round(mm["gemm2_TFLOPs"], 1) if mm["gemm2_TFLOPs"] else None,
                    "ffn_down_frac": round(mm["gemm2_TFLOPs"] / mm["peak"], 4) if mm["gemm2_TFLOPs"] else None,
                    "stage_ms": mm["stage_ms"], "stage_alone": mm["stage_alone"]})
            del tt
            torch.cuda.empty_cache()
        res["other_workloads"] = others
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
