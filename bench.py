#!/usr/bin/env python3
"""Benchmark of the MoE-layer hot path on one MI355X.

Default workload (the one the headline metric is quoted on): a step is one team_moe_layer_forward call
(router -> dispatch -> grouped SwiGLU FFN -> combine) over one block of 32 tokens of a 30B-A3B-shaped layer
(hidden 2048, 128 experts, top-8, intermediate 768, bf16) with routing confined to an activated-expert set of
M = 32 experts, inputs resident in HBM.  Consecutive steps rotate over several distinct weight sets so that no
weight byte is re-read before > 1 GB of other traffic (the 256 MB last-level cache would otherwise serve part
of a 151-302 MB working set).  The same loop is repeated for M in {128, 64, 32, 16} and reported under "sweep"
(step time vs number of activated experts).

Prints ONE JSON line.  `roofline` is for the expert FFN kernel (the one that streams the expert weights), timed
with HIP events on the launch stream around team_moe_expert_ffn; `cpu_baseline` is the CPU oracle on the same
workload on this machine's host cores.

Other workloads (--workload): cfg3 = 4 speculative candidates x 32 tokens sharing one set of 32 experts;
cfg5 = 256 tokens over 256 fine-grained experts (sets 256/96/48); cfg4 = a stack of 48 such layers run for 16
denoising steps with an activated set of 24 per (layer, step), a step being one pass over the whole stack;
block = the decoding of one 32-token block through that stack the way the paper's method runs it (live rows only, token
classes and the activated set decided on the device), next to the same block with every row and free routing.
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
MFMA_BF16_PEAK_TFLOPS = 2500.0
# HBM bytes per ffn_fused_kernel launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (see profiles/), keyed by
# (workload, activated-set size); counters cannot be read from inside this script.
PMC_TRAFFIC_BYTES = {("cfg2", 32): 306609997 + 2900434, ("cfg3", 32): 319283000 + 11553000, ("cfg5", 96): 625746000 + 20990000}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def run_block(args) -> int:
    """One diffusion block of 32 tokens decoded in 16 steps through a stack of MoE layers (MoE FFN only), two ways:
    (a) every step computes all 32 rows with free top-8 routing (no caching, no limited activation);
    (b) the paper's path: a step computes only the masked rows and the rows accepted in the previous step (Section "Delayed
        Caching for Decoded Tokens"), classes them on the device (Eq. 4, tau_h = 0.7, L_h = 3) and routes in two rounds
        (Algorithm 1), through team_moe_classify_tokens + team_moe_layer_forward_ex per layer.
    The acceptance schedule is synthetic and fixed (the two most confident masked positions per step, confidences drawn with a
    bias towards the left of the block: near-autoregressive decoding); it is input preparation, not part of the timed path."""
    import torch

    import paper_2602_08404_amd as tm
    from paper_2602_08404_amd import inputs as gen

    dev = "cuda:0"
    torch.cuda.set_device(0)
    shape = gen.CFG4
    L, H, E, k, I = shape.T, shape.H, shape.E, shape.k, shape.I
    n_layers = args.copies if args.copies > 0 else 48
    n_steps, tau_h, l_h = 16, 0.7, 3
    cfg = tm.make_config(H, I, E, k, "bf16", 1, L)

    def dev_t(a):
        return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)

    t0 = time.time()
    layers = []
    for c in range(n_layers):
        w = gen.make_weights(shape, seed=0, layer=c)
        layers.append(({n: dev_t(a) for n, a in w.items()},
                       [dev_t(gen.make_x(shape, seed=0, layer=c, step=st, kind=args.block_x, noise_std=0.40 if args.block_x == "structured" else 0.0552))
                        for st in range(n_steps)]))
        del w
    log(f"[bench] block: generated {n_layers} layers in {time.time() - t0:.1f}s")
    # ---- the schedule: state 0 masked, 2 accepted in the previous step (still computed), 1 decoded earlier (cached)
    state = np.zeros(L, np.uint8)
    sched = []
    for st in range(n_steps):
        conf = gen.confidences(L, seed=100 + st) ** (0.25 + 3.0 * np.arange(L) / L).astype(np.float32)
        live = np.nonzero(state != 1)[0].astype(np.int32)
        sched.append((torch.from_numpy(conf.astype(np.float32)).to(dev), torch.from_numpy(state.copy()).to(dev), torch.from_numpy(live).to(dev),
                      int(live.size)))
        state[state == 2] = 1
        masked = np.nonzero(state == 0)[0]
        take = masked[np.argsort(-conf[masked], kind="stable")[:2]]
        state[take] = 2
    ws = torch.empty(tm.team_moe_workspace_size(cfg), dtype=torch.uint8, device=dev)
    y = torch.empty((L, H), dtype=torch.bfloat16, device=dev)
    cls = torch.zeros((L,), dtype=torch.uint8, device=dev)
    e_a = torch.zeros((E,), dtype=torch.uint8, device=dev)
    n_a = torch.zeros((n_steps * n_layers,), dtype=torch.int32, device=dev)

    def block_all_rows():
        for st in range(n_steps):
            for d_w, xs in layers:
                tm.team_moe_layer_forward(cfg, xs[st], L, d_w["router"], d_w["gate"], d_w["up"], d_w["down"], None, y, ws)

    def block_team():
        for st in range(n_steps):
            conf, state_d, live, n_live = sched[st]
            tm.team_moe_classify_tokens(conf, state_d, L, L, live, n_live, tau_h, l_h, cls)
            for li, (d_w, xs) in enumerate(layers):
                tm.team_moe_layer_forward_ex(cfg, xs[st], y, n_live, d_w["router"], d_w["gate"], d_w["up"], d_w["down"], ws, row_index=live,
                                             n_rows=L, token_class=cls, activated_mask_out=e_a,
                                             n_activated_out=n_a[st * n_layers + li: st * n_layers + li + 1])

    def timed(fn, n):
        fn()
        torch.cuda.synchronize()
        t_begin = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t_begin) / n

    reps = max(1, args.steps // 100)
    s_all, s_team = timed(block_all_rows, reps), timed(block_team, reps)
    apf = n_a.cpu().numpy().reshape(n_steps, n_layers)
    live_counts = [c[3] for c in sched]
    log(f"[bench] block of {L} tokens, {n_steps} steps, {n_layers} layers: all rows + free routing {s_all * 1e3:.2f} ms; "
        f"live rows + two-round routing {s_team * 1e3:.2f} ms ({s_all / s_team:.2f}x); activated experts per layer call {apf.mean():.1f}")
    out = {"metric": "moe_layer_tokens_per_s", "value": L / s_team, "unit": "tokens/s", "n_gpus": 1, "steps": reps, "warmup": 1,
           "ms_per_step": s_team * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": f"block: one {L}-token block decoded in {n_steps} steps through {n_layers} cfg2-shaped MoE layers; a step of "
                                  "this line is the whole block (classification + two-round routing over the live rows, every layer, every step)",
                      "tokens": L, "layers": n_layers, "denoising_steps": n_steps, "tau_h": tau_h, "L_h": l_h, "hidden_states": args.block_x},
           "roofline": None, "cpu_baseline": None,
           "block": {"ms_all_rows_free_routing": s_all * 1e3, "ms_live_rows_two_round": s_team * 1e3, "speedup": s_all / s_team,
                     "live_rows_per_step": live_counts, "activated_per_layer_call_mean": float(apf.mean()),
                     "activated_per_step_mean": [float(v) for v in apf.mean(axis=1)],
                     "us_per_layer_call_all_rows": s_all * 1e6 / (n_steps * n_layers),
                     "us_per_layer_call_team": s_team * 1e6 / (n_steps * n_layers)}}
    print(json.dumps(out), flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", choices=["cfg2", "cfg3", "cfg4", "cfg5", "block"], default="cfg2")
    ap.add_argument("--copies", type=int, default=0, help="distinct weight sets rotated over (default 4; cfg4: layers of the stack, default 48)")
    ap.add_argument("--masks", type=str, default="",
                    help="activated-set sizes of the sweep (the headline size is always measured); e.g. --masks 32 for a profile of the headline only")
    ap.add_argument("--w8", action="store_true",
                    help="time the layer on 8-bit expert weights (E4M3 codes + row scales) instead of bf16 weights (not the headline)")
    ap.add_argument("--block-x", choices=["structured", "drift"], default="structured",
                    help="block workload: hidden states with a component shared by the rows of the block (default), or independent rows")
    ap.add_argument("--tokens", type=int, default=0,
                    help="cfg2 / cfg5 only: another number of tokens per call than the configuration's (a look beyond the listed workloads)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one process, one MI355X); --gpus must be 1. "
              "Nothing here uses a second GPU.", file=sys.stderr)
        return 2

    import torch

    import paper_2602_08404_amd as tm
    from paper_2602_08404_amd import inputs as gen

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.workload == "block":
        return run_block(args)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    wl = args.workload
    shape, x_kind, x_noise, default_masks, headline = {
        "cfg2": (gen.CFG2, "iid", 0.0, (128, 64, 32, 16), 32),
        "cfg3": (gen.CFG3, "candidates", 0.1, (32,), 32),
        "cfg4": (gen.CFG4, "drift", 0.0552, (24,), 24),
        "cfg5": (gen.CFG5, "iid", 0.0, (256, 96, 48), 96),
    }[wl]
    if args.tokens > 0:
        assert wl in ("cfg2", "cfg5") and args.tokens <= 1024, "--tokens: cfg2 / cfg5, at most 1024 tokens per call"
        shape = gen.scaled(shape, T=args.tokens)
    mask_sizes = tuple(sorted({int(v) for v in args.masks.split(",") if v} | {headline}, reverse=True)) if args.masks else default_masks
    T, H, E, k, I = shape.T, shape.H, shape.E, shape.k, shape.I
    A = T * k
    cfg = tm.make_config(H, I, E, k, "bf16", 1, T)
    bytes_per_expert = shape.bytes_per_expert
    n_sets = args.copies if args.copies > 0 else (48 if wl == "cfg4" else 4)
    n_steps_per_block = 16 if wl == "cfg4" else 1

    def dev_t(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(np.ascontiguousarray(a)).to(dev)

    ws = torch.empty(tm.team_moe_workspace_size(cfg), dtype=torch.uint8, device=dev)
    y = torch.empty((T, H), dtype=torch.bfloat16, device=dev)
    r_idx = torch.empty((T, k), dtype=torch.int32, device=dev)
    r_gate = torch.empty((T, k), dtype=torch.float32, device=dev)
    r_logits = torch.empty((T, E), dtype=torch.float32, device=dev)

    def gpu_logits(d_x, d_router):
        tm.team_moe_route(cfg, d_x, T, d_router, None, r_idx, r_gate, r_logits)
        torch.cuda.synchronize()
        return r_logits.cpu().numpy()

    # ---- inputs: weight sets (generator layers 0..n_sets-1); x per set (cfg4: per layer and denoising step);
    #      masks per (set, step, M) = top-M experts by summed router probability, from the GPU router's logits
    t0 = time.time()
    x_host0 = None
    host_w0 = None
    sets = []   # per set: (weights, [x per step], [masks per step: {M: tensor or None}])
    for c in range(n_sets):
        w = gen.make_weights(shape, seed=0, layer=c)
        d_w = {n: dev_t(a) for n, a in w.items()}
        xs, ms = [], []
        for step in range(n_steps_per_block):
            layer_for_x = c if wl == "cfg4" else 0
            xh = gen.make_x(shape, seed=0, layer=layer_for_x, step=step, kind=x_kind, noise_std=x_noise)
            if c == 0 and step == 0:
                x_host0, host_w0 = xh, w
            d_x = dev_t(xh)
            lg = gpu_logits(d_x, d_w["router"])
            xs.append(d_x)
            ms.append({M: (None if M == E else torch.from_numpy(gen.activated_set_by_summed_probability(lg, M)).to(dev)) for M in mask_sizes})
        sets.append((d_w, xs, ms))
        del w
    log(f"[bench] {wl}: generated {n_sets} weight sets in {time.time() - t0:.1f}s")

    stream = torch.cuda.current_stream()

    # ---- 8-bit copies of the expert weights (input preparation, on the device): the recipe of inputs.quantize_rows_e4m3 -
    #      scale = max|row| / 448 rounded to 8 significant bits, code = nearest E4M3 value of w / scale
    w8_supported = H in (1024, 2048) and I % 256 == 0
    sets_q = []

    def quantize_on_device(w_bf16):
        w = w_bf16.float()
        amax = w.abs().amax(dim=-1)
        scale = torch.where(amax > 0, amax / 448.0, torch.ones_like(amax)).bfloat16().float()
        q = (w / scale.unsqueeze(-1)).clamp_(-448.0, 448.0).to(torch.float8_e4m3fn).view(torch.uint8)
        return q.contiguous(), scale.contiguous()

    def w8_sets():
        if not sets_q:
            for c in range(n_sets):
                qs = {n: quantize_on_device(sets[c][0][n]) for n in ("gate", "up", "down")}
                sets_q.append(({n: v[0] for n, v in qs.items()}, {n: v[1] for n, v in qs.items()}))
            # same codes and scales as the host recipe (checked on one expert of set 0)
            wf = gen.as_f32(host_w0["down"][:1])
            code, sc = gen.quantize_rows_e4m3(wf)
            assert np.array_equal(sets_q[0][0]["down"][:1].cpu().numpy(), code) and np.array_equal(sets_q[0][1]["down"][:1].cpu().numpy(), sc)
        return sets_q

    def layer_w8(c, step, M):
        d_w, xs, ms = sets[c]
        q, sc = w8_sets()[c]
        tm.team_moe_layer_forward_w8(cfg, xs[step], T, d_w["router"], q["gate"], q["up"], q["down"], sc["gate"], sc["up"], sc["down"],
                                     ms[step][M], y, ws)

    def layer(c, step, M):
        if args.w8:
            return layer_w8(c, step, M)
        d_w, xs, ms = sets[c]
        tm.team_moe_layer_forward(cfg, xs[step], T, d_w["router"], d_w["gate"], d_w["up"], d_w["down"], ms[step][M], y, ws)

    def n_touched(c, step, M):
        """Experts that receive at least one token (their weights are what the call must read)."""
        d_w, xs, ms = sets[c]
        tm.team_moe_route(cfg, xs[step], T, d_w["router"], ms[step][M], r_idx, r_gate, None, ws)
        torch.cuda.synchronize()
        v = r_idx.cpu().numpy()
        return int(np.unique(v[v >= 0]).size)

    def bench_step(i, M):
        """One timed step: one layer call (cfg2/3/5, rotating weight sets) or one pass over the whole stack (cfg4)."""
        if wl == "cfg4":
            for c in range(n_sets):
                layer(c, i % n_steps_per_block, M)
        else:
            layer(i % n_sets, 0, M)

    def time_steps(M, steps, warmup):
        for i in range(warmup):
            bench_step(i, M)
        torch.cuda.synchronize()
        t_begin = time.perf_counter()
        for i in range(steps):
            bench_step(i, M)
        torch.cuda.synchronize()
        return (time.perf_counter() - t_begin) / steps

    # staged calls with HIP events around the expert FFN (same stream as the launches)
    st_off = torch.empty((E + 1,), dtype=torch.int32, device=dev)
    st_sorted = torch.empty((A,), dtype=torch.int32, device=dev)
    st_inv = torch.empty((T, k), dtype=torch.int32, device=dev)
    st_act = torch.empty((E,), dtype=torch.int32, device=dev)
    st_nact = torch.empty((1,), dtype=torch.int32, device=dev)
    st_out = torch.empty((A, H), dtype=torch.float32, device=dev)

    ffn_spread = {}          # (M, w8) -> (median, min) of the per-launch event times in ms

    def time_ffn(M, calls, warmup, w8=False):
        """Average duration of team_moe_expert_ffn (one launch of the weight-streaming kernel) from HIP events on the launch stream."""
        evs = []
        for i in range(warmup + calls):
            d_w, xs, ms = sets[i % n_sets]
            step = (i // n_sets) % n_steps_per_block
            tm.team_moe_route(cfg, xs[step], T, d_w["router"], ms[step][M], r_idx, r_gate, None, ws)
            tm.team_moe_build_dispatch(cfg, r_idx, T, st_off, st_sorted, st_inv, st_act, st_nact, ws)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            if w8:
                q, sc = w8_sets()[i % n_sets]
                e0.record(stream)
                tm.team_moe_expert_ffn_w8(cfg, xs[step], T, st_off, st_sorted, st_act, st_nact, q["gate"], q["up"], q["down"], sc["gate"],
                                          sc["up"], sc["down"], st_out, ws)
            else:
                e0.record(stream)
                tm.team_moe_expert_ffn(cfg, xs[step], T, st_off, st_sorted, st_act, st_nact, d_w["gate"], d_w["up"], d_w["down"], st_out, ws)
            e1.record(stream)
            tm.team_moe_combine(cfg, st_out, r_gate, st_inv, T, y)
            if i >= warmup:
                evs.append((e0, e1))
        torch.cuda.synchronize()
        ms = np.array([a.elapsed_time(b) for a, b in evs])
        ffn_spread[(M, w8)] = (float(np.median(ms)), float(ms.min()))
        return float(ms.mean()) * 1e-3

    def chunked_step_times(M, chunks=20, per_chunk=20):
        """Median and minimum over `chunks` groups of `per_chunk` back-to-back steps (seconds per step), outside the timed region."""
        times = []
        for c in range(chunks):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(per_chunk):
                bench_step(c * per_chunk + i, M)
            torch.cuda.synchronize()
            times.append((time.perf_counter() - t0) / per_chunk)
        return float(np.median(times)), float(np.min(times))

    # ---- headline: exactly `steps` timed steps between synchronisations
    if args.w8:
        assert w8_supported, "8-bit weights need hidden 1024 or 2048 and inter a multiple of 256"
        bytes_per_expert = 3 * H * I + (2 * I + H) * 4         # codes + row scales
    steps, warmup = (max(2, args.steps // 50), max(1, args.warmup // 20)) if wl == "cfg4" else (args.steps, args.warmup)
    sec_per_step = time_steps(headline, steps, warmup)
    layers_per_step = n_sets if wl == "cfg4" else 1
    sample_sets = range(min(n_sets, 4))
    touched = {M: float(np.mean([n_touched(c, 0, M) for c in sample_sets])) for M in mask_sizes}
    sweep = []
    for M in mask_sizes:
        s_step = sec_per_step if M == headline else time_steps(M, max(50, steps // 2), max(10, warmup // 2))
        s_layer = s_step / layers_per_step
        s_ffn = time_ffn(M, max(50, args.steps // 2), max(10, args.warmup // 2), w8=args.w8)
        wbytes = touched[M] * bytes_per_expert
        flops = 2.0 * A * 3 * H * I
        sweep.append({"activated": M, "touched": touched[M], "ms_per_layer": s_layer * 1e3, "tokens_per_s": T / s_step,
                      "ffn_ms": s_ffn * 1e3, "ffn_ms_median": ffn_spread[(M, args.w8)][0], "ffn_ms_min": ffn_spread[(M, args.w8)][1],
                      "weight_GBps_ffn": wbytes / s_ffn / 1e9, "weight_GBps_layer": wbytes / s_layer / 1e9,
                      "ffn_TFLOPs": flops / s_ffn / 1e12, "mfma_frac": flops / s_ffn / 1e12 / MFMA_BF16_PEAK_TFLOPS})
        log(f"[bench] {wl} M={M}: layer {s_layer * 1e6:.1f} us, ffn {s_ffn * 1e6:.1f} us, touched {touched[M]:.1f}, "
            f"ffn weight stream {wbytes / s_ffn / 1e9:.0f} GB/s, {flops / s_ffn / 1e12:.1f} TFLOP/s")
    head = next(r for r in sweep if r["activated"] == headline)
    roofline = {"bound": "hbm", "kernel": "ffn_fused_kernel (team_moe_expert_ffn: gate/up + down GEMMs of the activated experts, one launch)",
                "achieved": head["weight_GBps_ffn"], "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": head["weight_GBps_ffn"] / HBM_PEAK_GBS,
                "traffic": PMC_TRAFFIC_BYTES.get((wl, headline)), "bytes_per_launch": touched[headline] * bytes_per_expert,
                "launch_us": head["ffn_ms"] * 1e3}

    # ---- the same layer with the activated set decided on the device (Algorithm 1: two-round routing from token classes)
    two_round = None
    if wl != "cfg4" and not args.masks:                      # left out of the headline-only runs used for profiles
        n_first = max(1, T // 8)
        cls = [torch.from_numpy(gen.token_classes(T, n_first, seed=c)).to(dev) for c in range(n_sets)]
        d_nact = torch.zeros((1,), dtype=torch.int32, device=dev)
        d_mask = torch.zeros((E,), dtype=torch.uint8, device=dev)

        def layer2(i):
            d_w, xs, ms = sets[i % n_sets]
            tm.team_moe_layer_forward_two_round(cfg, xs[0], T, d_w["router"], d_w["gate"], d_w["up"], d_w["down"], cls[i % n_sets],
                                                d_mask, d_nact, y, ws)

        n_act = []
        for c in range(n_sets):
            layer2(c)
            torch.cuda.synchronize()
            n_act.append(int(d_nact.item()))
        n2 = max(50, steps // 2)
        for i in range(10):
            layer2(i)
        torch.cuda.synchronize()
        t_begin = time.perf_counter()
        for i in range(n2):
            layer2(i)
        torch.cuda.synchronize()
        s2 = (time.perf_counter() - t_begin) / n2
        two_round = {"first_round_tokens": n_first, "activated": float(np.mean(n_act)), "ms_per_layer": s2 * 1e3, "tokens_per_s": T / s2}
        log(f"[bench] {wl} two-round routing: {n_first} first-round tokens -> |E_A| = {np.mean(n_act):.1f}, layer {s2 * 1e6:.1f} us")

    # ---- the headline workload on 8-bit expert weights (half the weight bytes; a variant outside the paper)
    w8 = None
    if wl == "cfg2" and w8_supported and not args.masks and not args.w8:
        def timed_w8(n):
            for i in range(10):
                layer_w8(i % n_sets, 0, headline)
            torch.cuda.synchronize()
            t_begin = time.perf_counter()
            for i in range(n):
                layer_w8(i % n_sets, 0, headline)
            torch.cuda.synchronize()
            return (time.perf_counter() - t_begin) / n

        s8 = timed_w8(max(50, steps // 2))
        f8 = time_ffn(headline, max(50, args.steps // 2), 10, w8=True)
        b8 = touched[headline] * (3 * H * I + (2 * I + H) * 4)
        w8 = {"weights": "E4M3 codes + one float scale per row", "activated": headline, "ms_per_layer": s8 * 1e3, "tokens_per_s": T / s8,
              "ffn_ms": f8 * 1e3, "weight_bytes_per_launch": b8, "weight_GBps_ffn": b8 / f8 / 1e9, "frac_of_hbm_peak": b8 / f8 / 1e9 / HBM_PEAK_GBS}
        log(f"[bench] {wl} M={headline} on 8-bit weights: layer {s8 * 1e6:.1f} us, ffn {f8 * 1e6:.1f} us, weight stream {b8 / f8 / 1e9:.0f} GB/s")

    # ---- candidate branches with repeated rows (Section "Aligned Token Candidates in SEH"): the same layer over 4 x 32 rows of
    #      which 34 are distinct, computed row by row and with every distinct row computed once
    branches = None
    if wl == "cfg3" and not args.masks:
        bx, bm = [], []
        for c in range(n_sets):
            d_x = dev_t(gen.make_x(shape, seed=0, layer=0, step=c, kind="branches"))
            bx.append(d_x)
            bm.append(torch.from_numpy(gen.activated_set_by_summed_probability(gpu_logits(d_x, sets[c][0]["router"]), headline)).to(dev))
        d_rep = torch.zeros((T,), dtype=torch.int32, device=dev)
        d_nu = torch.zeros((1,), dtype=torch.int32, device=dev)

        def plain(i):
            d_w = sets[i % n_sets][0]
            tm.team_moe_layer_forward(cfg, bx[i % n_sets], T, d_w["router"], d_w["gate"], d_w["up"], d_w["down"], bm[i % n_sets], y, ws)

        def unique(i):
            d_w = sets[i % n_sets][0]
            tm.team_moe_layer_forward_unique_rows(cfg, bx[i % n_sets], T, d_w["router"], d_w["gate"], d_w["up"], d_w["down"],
                                                  bm[i % n_sets], y, d_rep, d_nu, ws)

        def timed(fn, n):
            for i in range(10):
                fn(i)
            torch.cuda.synchronize()
            t_begin = time.perf_counter()
            for i in range(n):
                fn(i)
            torch.cuda.synchronize()
            return (time.perf_counter() - t_begin) / n

        nb = max(50, steps // 2)
        s_plain, s_unique = timed(plain, nb), timed(unique, nb)
        n_unique = int(d_nu.item())
        branches = {"rows": T, "distinct_rows": n_unique, "rows_per_expert": A / headline, "distinct_rows_per_expert": n_unique * k / headline,
                    "ms_per_layer_all_rows": s_plain * 1e3, "ms_per_layer_distinct_rows": s_unique * 1e3,
                    "tokens_per_s_all_rows": T / s_plain, "tokens_per_s_distinct_rows": T / s_unique}
        log(f"[bench] cfg3 branches with repeated rows: {n_unique} distinct of {T}; layer {s_plain * 1e6:.1f} us row by row, "
            f"{s_unique * 1e6:.1f} us with distinct rows computed once")

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

    # ---- CPU baseline: the oracle, as it stands, on the same workload (weight set 0, headline M), host cores of this machine
    cpu = None
    if not args.no_cpu:
        from oracle import c_oracle as orc
        wf = {n: gen.as_f32(a) for n, a in host_w0.items()}
        xf = gen.as_f32(x_host0)
        mask = gen.activated_set_by_summed_probability(orc.router_logits(xf, wf["router"]), headline)
        orc.moe_layer(xf, wf["router"], wf["gate"], wf["up"], wf["down"], k, 1, mask)          # warm
        n, t_begin = 0, time.perf_counter()
        while time.perf_counter() - t_begin < args.cpu_seconds:
            orc.moe_layer(xf, wf["router"], wf["gate"], wf["up"], wf["down"], k, 1, mask)
            n += 1
        el = time.perf_counter() - t_begin
        cpu_tokens_per_s = T * n / el / layers_per_step          # cfg4: a token has passed the step when all layers are done
        cpu = {"value": cpu_tokens_per_s, "unit": "tokens/s", "cores": orc.max_threads(), "kind": "oracle",
               "sample": f"{n} single-layer calls of the same workload (weight set 0, M={headline}, {T} tokens each) in {el:.1f}s"
                         + (f"; scaled to the {layers_per_step}-layer step" if layers_per_step > 1 else "")}

    desc = {
        "cfg2": f"cfg2: one 30B-A3B-shaped MoE layer (H=2048, E=128, top-8, I=768, bf16), block of 32 tokens, activated-expert set "
                f"M={headline} (top experts by summed router probability), {n_sets} weight sets rotated",
        "cfg3": f"cfg3: same layer, 4 speculative candidates x 32 tokens = 128 tokens sharing one activated set of {headline} experts, "
                f"{n_sets} weight sets rotated",
        "cfg4": f"cfg4: stack of {n_sets} cfg2 layers (MoE FFN only), one 32-token block, 16 denoising steps with drifting hidden states, "
                f"activated set of {headline} per (layer, step); a step = one pass over the stack",
        "cfg5": f"cfg5: fine-grained layer (H=2048, E=256, top-8, I=512, bf16), 256 tokens, activated set M={headline}, {n_sets} weight sets rotated",
    }[wl]
    if args.tokens > 0:
        desc = f"{wl} shape at {T} tokens per call instead of the configuration's (not a listed workload): " + desc
    out = {"metric": "moe_layer_tokens_per_s", "value": T / sec_per_step, "unit": "tokens/s", "n_gpus": 1, "steps": steps,
           "warmup": warmup, "ms_per_step": sec_per_step * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "bf16", "data": "synthetic" + (" (expert weights stored as E4M3 codes with row scales)" if args.w8 else ""),
           "config": {"workload": desc, "tokens": T, "activated": headline, "touched": touched[headline], "layers_per_step": layers_per_step},
           "roofline": roofline, "cpu_baseline": cpu, "sweep": sweep, "two_round": two_round, "branches": branches, "w8": w8,
           "device_copy_GBps": copy_gbps}
    if wl == "cfg4":
        out["ms_per_block_16_steps"] = sec_per_step * 1e3 * 16
    else:
        med, mn = chunked_step_times(headline)
        out["ms_per_step_median"], out["ms_per_step_min"] = med * 1e3, mn * 1e3
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
