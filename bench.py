#!/usr/bin/env python3
"""Benchmark of the ETR MoE-layer forward on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config cfg2] [--capacity C] [--no-cpu-baseline]

A "step" is one pass of the whole hot path (route -> select -> dispatch -> expert FFN ->
combine, one etr_moe_forward call) over one batch of seeded synthetic tokens that is
already resident in HBM.  Prints ONE JSON line: tokens/s of the whole layer, the roofline
position of the dominant kernel (the gate/up MFMA grouped GEMM) measured with HIP events
on the launch stream, per-stage times, and the CPU oracle timed on a bounded sample.
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
PEAK_F32_TFLOPS = 157.3       # fp32 vector
PEAK_HBM_GBS = 8000.0

# HBM bytes per launch of the dominant kernel (FFN gate/up GEMM), measured with rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE on this very command and scaled by what a plain 1 GiB copy reads on the same counters (fetch x2.0,
# write x1.0); the summaries are profiles/moe_forward_<cfg>_kernels_and_traffic.txt. None = not measured.
MEASURED_TRAFFIC_BYTES = {"cfg2": 1034.2e6 + 136.6e6, "cfg5": 13652.0e6 + 719.5e6}


def _to_np(t):
    import numpy as np
    import torch
    t = t.detach().cpu().contiguous()
    return t.view(torch.int16).numpy().view(np.uint16) if t.dtype == torch.bfloat16 else t.numpy()


def cpu_baseline(shape, cfg, tensors, budget_tokens: int):
    """Times the oracle (as it stands) on the host cores: routing on all T tokens, the expert
    FFN and the weighted sum on the first `budget_tokens` tokens, extrapolated linearly in tokens."""
    import numpy as np
    from oracle import etr_ref
    host = {k: _to_np(v) for k, v in tensors.items()}
    n = min(budget_tokens, shape.T)
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
    return {"value": shape.T / t_full, "unit": "tokens/s", "cores": etr_ref.num_threads(), "kind": "oracle",
            "sample": f"routing on all {shape.T} tokens ({t_routing:.2f} s); FFN+combine on the first {n} tokens "
                      f"({t_sample - t_routing:.2f} s), extrapolated linearly to {shape.T}"}


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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="cfg2")
    ap.add_argument("--capacity", type=int, default=None, help="override the capacity (cfg4's schedule)")
    ap.add_argument("--cpu-tokens", type=int, default=8192, help="tokens of the oracle's FFN sample")
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
    out = torch.empty(shape.T, shape.d, dtype=shape.torch_dtype, device=dev)
    counts = torch.zeros(shape.E, dtype=torch.int32, device=dev)
    if args.backward:
        return bench_backward(args, shape, cfg, t, dev)
    ws = B.alloc_workspace(B.etr_workspace_bytes(cfg), dev)

    def step(events=None):
        if events is None:
            B.etr_moe_forward(cfg, t["x"], t["w_emb"], t["w_gate"], t["w_up"], t["w_down"], out, ws, counts=counts)
        else:
            B.etr_moe_forward_profiled(cfg, t["x"], t["w_emb"], t["w_gate"], t["w_up"], t["w_down"], out, ws, events,
                                       counts=counts)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # timed region: K steps; only the dominant kernel (FFN gate/up GEMM) is bracketed by events
    # (boundaries 3 and 4), because every recorded event costs a few microseconds of stream time
    gemm_events = [B.StageEvents(only=(3, 4)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(gemm_events[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    t_gemm1_ms = sum(B.elapsed_ms(ev, 3, 4) for ev in gemm_events) / args.steps
    # second pass, all stage boundaries marked: the per-stage breakdown (not part of `value`)
    events = [B.StageEvents() for _ in range(args.steps)]
    for i in range(args.steps):
        step(events[i])
    torch.cuda.synchronize()

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

    ms_per_step = 1e3 * elapsed / args.steps
    stage = [0.0] * (B.N_STAGE_EVENTS - 1)
    for ev in events:
        for i, ms in enumerate(ev.stage_ms()):
            stage[i] += ms / args.steps
    rows = int(counts.sum().item())
    elt = 4 if shape.dtype == I.DT_F32 else 2
    # dominant kernel: FFN GEMM-1 (gate and up projections + SwiGLU), 4*d*H flop per kept row
    flops_gemm1 = 4.0 * rows * shape.d * shape.H
    t_gemm1 = t_gemm1_ms * 1e-3
    peak = PEAK_BF16_TFLOPS if shape.dtype == I.DT_BF16 else PEAK_F32_TFLOPS
    achieved = flops_gemm1 / t_gemm1 / 1e12
    stages = {name: round(ms, 5) for name, ms in zip(B.STAGE_NAMES, stage)}
    # algorithmic bytes of the HBM-bound stages -> GB/s (for the report; the roofline object is the GEMM's)
    TE = shape.T * shape.E
    bytes_alg = {
        "route": shape.T * shape.d * elt + 2 * TE * 4,
        "dispatch": rows * (2 * shape.d * elt + 4),
        "combine": rows * shape.d * elt + shape.T * shape.d * elt + TE * 8,
    }
    hbm = {k: {"us": round(alone[k] * 1e3, 2), "GBs": round(v / (alone[k] * 1e-3) / 1e9, 1),
               "frac_of_8TBs": round(v / (alone[k] * 1e-3) / 1e9 / PEAK_HBM_GBS, 3)} for k, v in bytes_alg.items()}
    hbm["select"] = {"us": round(alone["select"] * 1e3, 2)}
    flops_gemm2 = 2.0 * rows * shape.d * shape.H
    res = {
        "metric": "MoE-layer tokens/sec on 1 MI355X",
        "value": shape.T / (elapsed / args.steps),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if shape.dtype == I.DT_BF16 else "f32",
        "data": "synthetic",
        "config": {"workload": f"{shape.name}: T={shape.T} d={shape.d} E={shape.E} D={shape.D} k={shape.k} "
                               f"capacity={cfg.capacity} H={shape.H} mode={('TCR', 'ECR', 'BIDIR')[cfg.mode]} "
                               f"tokens={shape.recipe}",
                   "kept_rows": rows},
        "roofline": {"kernel": "gemm_bf16_persist64_kernel<GLU> (FFN gate/up projections + SwiGLU)"
                     if shape.dtype == I.DT_BF16 else "gemm_f32_kernel<GLU>",
                     "bound": "mfma" if shape.dtype == I.DT_BF16 else "alu",
                     "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(args.config) if args.capacity is None else None,
                     "algorithmic_flop": flops_gemm1,
                     "algorithmic_bytes": elt * (2.0 * shape.E * shape.H * shape.d + rows * shape.d
                                                 + rows * shape.H)},
        "stage_ms": stages,
        "stage_alone": hbm,
        "ffn_down_TFLOPs": flops_gemm2 / (stage[4] * 1e-3) / 1e12 if stage[4] > 0 else None,
    }
    if args.calibrate_copy:
        a = torch.ones(1 << 30, dtype=torch.uint8, device=dev)
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(shape, cfg, t, args.cpu_tokens)
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
