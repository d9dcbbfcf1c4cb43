#!/usr/bin/env python3
"""Benchmark of the MoE-layer hot path on one MI355X.

A step is one team_moe_layer_forward call (router -> dispatch -> grouped SwiGLU FFN -> combine) over one block
of 32 tokens of a 30B-A3B-shaped layer (hidden 2048, 128 experts, top-8, intermediate 768, bf16) with routing
confined to an activated-expert set of M = 32 experts, inputs resident in HBM.  Consecutive steps rotate over
several distinct weight sets so that no weight byte is re-read before > 1 GB of other traffic (the 256 MB
last-level cache would otherwise serve part of a 151-302 MB working set).  The same loop is repeated for
M in {128, 64, 32, 16} and reported under "sweep" (step time vs number of activated experts).

Prints ONE JSON line.  `roofline` is for the expert FFN (the kernels that stream the expert weights), timed
with HIP events on the launch stream around team_moe_expert_ffn; `cpu_baseline` is the CPU oracle on the same
workload on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MASK_SIZES = (128, 64, 32, 16)
HEADLINE_M = 32


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--copies", type=int, default=4, help="distinct weight sets rotated over")
    ap.add_argument("--masks", type=str, default="128,64,32,16",
                    help="activated-set sizes of the sweep (the headline size 32 is always measured); e.g. --masks 32 for a profile of the headline only")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one process, one MI355X); --gpus must be 1. "
              "Nothing here uses a second GPU.", file=sys.stderr)
        return 2

    global MASK_SIZES
    MASK_SIZES = tuple(sorted({int(v) for v in args.masks.split(",") if v} | {HEADLINE_M}, reverse=True))

    import torch

    import paper_2602_08404_amd as tm
    from paper_2602_08404_amd import inputs as gen

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    shape = gen.CFG2
    T, H, E, k, I = shape.T, shape.H, shape.E, shape.k, shape.I
    cfg = tm.make_config(H, I, E, k, "bf16", 1, T)
    bytes_per_expert = shape.bytes_per_expert

    def dev_t(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(np.ascontiguousarray(a)).to(dev)

    # ---- inputs: one x, `copies` weight sets (generator layers 0..copies-1), masks per (copy, M) from the GPU router's logits
    x_host = gen.make_x(shape, seed=0)
    d_x = dev_t(x_host)
    ws = torch.empty(tm.team_moe_workspace_size(cfg), dtype=torch.uint8, device=dev)
    y = torch.empty((T, H), dtype=torch.bfloat16, device=dev)
    copies = []
    host_w0 = None
    t0 = time.time()
    for c in range(args.copies):
        w = gen.make_weights(shape, seed=0, layer=c)
        if c == 0:
            host_w0 = w
        d_w = {n: dev_t(a) for n, a in w.items()}
        idx = torch.empty((T, k), dtype=torch.int32, device=dev)
        gate = torch.empty((T, k), dtype=torch.float32, device=dev)
        logits = torch.empty((T, E), dtype=torch.float32, device=dev)
        tm.team_moe_route(cfg, d_x, T, d_w["router"], None, idx, gate, logits)
        torch.cuda.synchronize()
        lg = logits.cpu().numpy()
        masks = {M: (None if M == E else torch.from_numpy(gen.activated_set_by_summed_probability(lg, M)).to(dev)) for M in MASK_SIZES}
        copies.append((d_w, masks))
        del w
    log(f"[bench] generated {args.copies} weight sets in {time.time() - t0:.1f}s")

    stream = torch.cuda.current_stream()

    def layer(c, M):
        d_w, masks = copies[c]
        tm.team_moe_layer_forward(cfg, d_x, T, d_w["router"], d_w["gate"], d_w["up"], d_w["down"], masks[M], y, ws)

    def n_touched(c, M):
        """Experts that receive at least one token (their weights are what the call must read)."""
        d_w, masks = copies[c]
        idx = torch.empty((T, k), dtype=torch.int32, device=dev)
        gate = torch.empty((T, k), dtype=torch.float32, device=dev)
        tm.team_moe_route(cfg, d_x, T, d_w["router"], masks[M], idx, gate, None, ws)
        torch.cuda.synchronize()
        v = idx.cpu().numpy()
        return int(np.unique(v[v >= 0]).size)

    def time_layer(M, steps, warmup):
        for i in range(warmup):
            layer(i % args.copies, M)
        torch.cuda.synchronize()
        t_begin = time.perf_counter()
        for i in range(steps):
            layer(i % args.copies, M)
        torch.cuda.synchronize()
        return (time.perf_counter() - t_begin) / steps

    # staged calls with HIP events around the expert FFN (same stream as the launches)
    A = T * k
    st_idx = torch.empty((T, k), dtype=torch.int32, device=dev)
    st_gate = torch.empty((T, k), dtype=torch.float32, device=dev)
    st_off = torch.empty((E + 1,), dtype=torch.int32, device=dev)
    st_sorted = torch.empty((A,), dtype=torch.int32, device=dev)
    st_inv = torch.empty((T, k), dtype=torch.int32, device=dev)
    st_act = torch.empty((E,), dtype=torch.int32, device=dev)
    st_nact = torch.empty((1,), dtype=torch.int32, device=dev)
    st_out = torch.empty((A, H), dtype=torch.float32, device=dev)

    def time_ffn(M, steps, warmup):
        """Average duration of team_moe_expert_ffn (the weight-streaming kernels) from HIP events on the launch stream."""
        evs = []
        for i in range(warmup + steps):
            d_w, masks = copies[i % args.copies]
            tm.team_moe_route(cfg, d_x, T, d_w["router"], masks[M], st_idx, st_gate, None, ws)
            tm.team_moe_build_dispatch(cfg, st_idx, T, st_off, st_sorted, st_inv, st_act, st_nact, ws)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            tm.team_moe_expert_ffn(cfg, d_x, T, st_off, st_sorted, st_act, st_nact, d_w["gate"], d_w["up"], d_w["down"], st_out, ws)
            e1.record(stream)
            tm.team_moe_combine(cfg, st_out, st_gate, st_inv, T, y)
            if i >= warmup:
                evs.append((e0, e1))
        torch.cuda.synchronize()
        return float(np.mean([a.elapsed_time(b) for a, b in evs])) * 1e-3

    # ---- headline: M = 32, exactly `steps` timed steps between synchronisations
    sec_per_step = time_layer(HEADLINE_M, args.steps, args.warmup)
    touched = {M: float(np.mean([n_touched(c, M) for c in range(args.copies)])) for M in MASK_SIZES}
    sweep = []
    for M in MASK_SIZES:
        s_layer = sec_per_step if M == HEADLINE_M else time_layer(M, max(50, args.steps // 2), max(10, args.warmup // 2))
        s_ffn = time_ffn(M, max(50, args.steps // 2), max(10, args.warmup // 2))
        wbytes = touched[M] * bytes_per_expert
        sweep.append({"activated": M, "touched": touched[M], "ms_per_step": s_layer * 1e3, "tokens_per_s": T / s_layer,
                      "ffn_ms": s_ffn * 1e3, "weight_GBps_ffn": wbytes / s_ffn / 1e9, "weight_GBps_layer": wbytes / s_layer / 1e9})
        log(f"[bench] M={M}: layer {s_layer * 1e6:.1f} us, ffn {s_ffn * 1e6:.1f} us, touched {touched[M]:.1f}, "
            f"ffn weight stream {wbytes / s_ffn / 1e9:.0f} GB/s")
    head = next(r for r in sweep if r["activated"] == HEADLINE_M)
    roofline = {"bound": "hbm", "kernel": "ffn_fused_kernel (team_moe_expert_ffn: gate/up + down GEMMs of the activated experts, one launch)",
                "achieved": head["weight_GBps_ffn"], "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": head["weight_GBps_ffn"] / HBM_PEAK_GBS,
                "traffic": None, "bytes_per_launch": touched[HEADLINE_M] * bytes_per_expert}

    # ---- context: plain device-to-device copy rate (read + write bytes) of 1 GiB, the practical streaming ceiling
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record(stream)
    for _ in range(10):
        dst.copy_(src)
    c1.record(stream)
    torch.cuda.synchronize()
    copy_gbps = 2.0 * src.numel() * 10 / (c0.elapsed_time(c1) * 1e-3) / 1e9
    del src, dst

    # ---- CPU baseline: the oracle, as it stands, on the same workload (copy 0, M = 32), host cores of this machine
    cpu = None
    if not args.no_cpu:
        from oracle import c_oracle as orc
        wf = {n: gen.as_f32(a) for n, a in host_w0.items()}
        xf = gen.as_f32(x_host)
        mask = gen.activated_set_by_summed_probability(orc.router_logits(xf, wf["router"]), HEADLINE_M)
        orc.moe_layer(xf, wf["router"], wf["gate"], wf["up"], wf["down"], k, 1, mask)          # warm
        n, t_begin = 0, time.perf_counter()
        while time.perf_counter() - t_begin < args.cpu_seconds:
            orc.moe_layer(xf, wf["router"], wf["gate"], wf["up"], wf["down"], k, 1, mask)
            n += 1
        el = time.perf_counter() - t_begin
        cpu = {"value": T * n / el, "unit": "tokens/s", "cores": orc.max_threads(), "kind": "oracle",
               "sample": f"{n} full layer calls of the same workload (weight set 0, M={HEADLINE_M}, 32 tokens each) in {el:.1f}s"}

    out = {"metric": "moe_layer_tokens_per_s", "value": T / sec_per_step, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": sec_per_step * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "bf16", "data": "synthetic",
           "config": {"workload": f"cfg2: one 30B-A3B-shaped MoE layer (H=2048, E=128, top-8, I=768, bf16), block of 32 tokens, "
                                  f"activated-expert set M={HEADLINE_M} (top experts by summed router probability), "
                                  f"{args.copies} weight sets rotated", "tokens": T, "activated": HEADLINE_M,
                      "touched": touched[HEADLINE_M]},
           "roofline": roofline, "cpu_baseline": cpu, "sweep": sweep, "device_copy_GBps": copy_gbps}
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
