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
with HIP events that the library records on the launch stream directly before and after that kernel inside the
layer call; `cpu_baseline` is the CPU oracle on the same workload on this machine's host cores (all cores, and one
thread); `parity` is one timed call's output checked against the oracle; `workloads` repeats layer time, FFN kernel
time, roofline fraction and parity for the other listed configurations (cfg3, cfg4 on 8 of its 48 independent layers,
cfg5); `ceilings` are a device copy and a read-only stream of the sizes the FFN streams, measured in the same run.

Single workloads (--workload cfgN: that workload as the headline, for profiles): cfg3 = 4 speculative candidates x 32 tokens sharing one set of 32 experts;
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
# HBM bytes per ffn_fused_kernel launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE and the file under profiles/ that holds the
# counter runs, keyed by (workload, activated-set size); counters cannot be read from inside this script.
PMC_TRAFFIC = {("cfg2", 32): (306700000 + 2900000, "profiles/moe_layer_kernels_cfg2_M32.md"),
               ("cfg3", 32): (319400000 + 11600000, "profiles/expert_ffn_cfg3_cfg4_cfg5.md"),
               ("cfg5", 96): (625800000 + 21000000, "profiles/expert_ffn_cfg3_cfg4_cfg5.md")}


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


# ----------------------------------------------------------------------------------------------------------------------------
WORKLOADS = {
    #        shape attr  x kind        noise    activated-set sizes   headline
    "cfg2": ("CFG2", "iid",        0.0,    (128, 64, 32, 16), 32),
    "cfg3": ("CFG3", "candidates", 0.1,    (32,),             32),
    "cfg4": ("CFG4", "drift",      0.0552, (24,),             24),
    "cfg5": ("CFG5", "iid",        0.0,    (256, 96, 48),     96),
}
PARITY_BAR = 2e-2           # per row max|gpu - ref| / max|ref|, bf16 storage
GAP = 1e-4                  # tokens whose k-th / (k+1)-th allowed score are closer than this may select differently


class Workload:
    """One listed configuration on the device: weight sets rotated over, inputs, activated sets, and the timing loops."""

    def __init__(self, wl, args, torch, tm, gen, n_sets=None, tokens=0, mask_sizes=None):
        from oracle import c_oracle as orc              # the activated sets are drawn from the oracle's router scores (input recipe)
        self.wl, self.args, self.torch, self.tm, self.gen = wl, args, torch, tm, gen
        attr, self.x_kind, self.x_noise, default_masks, self.headline = WORKLOADS[wl]
        shape = getattr(gen, attr)
        if tokens > 0:
            shape = gen.scaled(shape, T=tokens)
        self.shape = shape
        self.mask_sizes = tuple(mask_sizes) if mask_sizes else default_masks
        T, H, E, k, I = shape.T, shape.H, shape.E, shape.k, shape.I
        self.T, self.H, self.E, self.k, self.I, self.A = T, H, E, k, I, T * k
        self.dev = dev = "cuda:0"
        self.cfg = tm.make_config(H, I, E, k, "bf16", 1, T)
        self.n_sets = n_sets or (8 if wl == "cfg4" else 4)
        self.steps_per_block = 16 if wl == "cfg4" else 1
        self.layers_per_step = self.n_sets if wl == "cfg4" else 1
        self.bytes_per_expert = shape.bytes_per_expert
        self.ws = torch.empty(tm.team_moe_workspace_size(self.cfg), dtype=torch.uint8, device=dev)
        self.y = torch.empty((T, H), dtype=torch.bfloat16, device=dev)
        self.r_idx = torch.empty((T, k), dtype=torch.int32, device=dev)
        self.r_gate = torch.empty((T, k), dtype=torch.float32, device=dev)
        self.stream = torch.cuda.current_stream()
        t0 = time.time()
        self.sets = []           # per set: (device weights, [x per step], [masks per step: {M: tensor or None}])
        self.host0 = None        # set 0, step 0 on the host, for the parity check and the CPU baseline
        for c in range(self.n_sets):
            w = gen.make_weights(shape, seed=0, layer=c)
            d_w = {n: self.dev_t(a) for n, a in w.items()}
            router_f32 = gen.as_f32(w["router"])
            xs, ms = [], []
            for step in range(self.steps_per_block):
                xh = gen.make_x(shape, seed=0, layer=c if wl == "cfg4" else 0, step=step, kind=self.x_kind, noise_std=self.x_noise)
                lg = orc.router_logits(gen.as_f32(xh), router_f32)
                masks_h = {M: (None if M == E else gen.activated_set_by_summed_probability(lg, M)) for M in self.mask_sizes}
                if c == 0 and step == 0:
                    self.host0 = (xh, w, masks_h, lg)
                xs.append(self.dev_t(xh))
                ms.append({M: (None if m is None else torch.from_numpy(m).to(dev)) for M, m in masks_h.items()})
            self.sets.append((d_w, xs, ms))
            del w
        log(f"[bench] {wl}: generated {self.n_sets} weight sets in {time.time() - t0:.1f}s")
        self.sets_q = []
        # two events per timed launch, reused: created once (torch makes the handle on the first record)
        self.ev = None

    def dev_t(self, a):
        torch = self.torch
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).to(self.dev).view(torch.bfloat16)
        return torch.from_numpy(np.ascontiguousarray(a)).to(self.dev)

    # ---- 8-bit copies of the expert weights (input preparation, on the device): the recipe of inputs.quantize_rows_e4m3
    def w8_supported(self):
        return self.H in (1024, 2048) and self.I % 256 == 0

    def w8_sets(self):
        torch, gen = self.torch, self.gen
        if not self.sets_q:
            def quantize_on_device(w_bf16):
                w = w_bf16.float()
                amax = w.abs().amax(dim=-1)
                scale = torch.where(amax > 0, amax / 448.0, torch.ones_like(amax)).bfloat16().float()
                q = (w / scale.unsqueeze(-1)).clamp_(-448.0, 448.0).to(torch.float8_e4m3fn).view(torch.uint8)
                return q.contiguous(), scale.contiguous()
            for c in range(self.n_sets):
                qs = {n: quantize_on_device(self.sets[c][0][n]) for n in ("gate", "up", "down")}
                self.sets_q.append(({n: v[0] for n, v in qs.items()}, {n: v[1] for n, v in qs.items()}))
            wf = gen.as_f32(self.host0[1]["down"][:1])          # same codes and scales as the host recipe (one expert of set 0)
            code, sc = gen.quantize_rows_e4m3(wf)
            assert np.array_equal(self.sets_q[0][0]["down"][:1].cpu().numpy(), code) and np.array_equal(self.sets_q[0][1]["down"][:1].cpu().numpy(), sc)
        return self.sets_q

    # ---- one layer call
    def layer(self, c, step, M, w8=False, events=None):
        tm = self.tm
        d_w, xs, ms = self.sets[c]
        if w8:
            q, sc = self.w8_sets()[c]
            tm.team_moe_layer_forward_ex(self.cfg, xs[step], self.y, self.T, d_w["router"], q["gate"], q["up"], q["down"], self.ws,
                                         scales=(sc["gate"], sc["up"], sc["down"]), expert_mask=ms[step][M], ffn_events=events)
        elif events is not None:
            tm.team_moe_layer_forward_ex(self.cfg, xs[step], self.y, self.T, d_w["router"], d_w["gate"], d_w["up"], d_w["down"], self.ws,
                                         expert_mask=ms[step][M], ffn_events=events)
        else:
            tm.team_moe_layer_forward(self.cfg, xs[step], self.T, d_w["router"], d_w["gate"], d_w["up"], d_w["down"], ms[step][M], self.y, self.ws)

    def n_touched(self, c, step, M):
        """Experts that receive at least one token (their weights are what the call must read)."""
        d_w, xs, ms = self.sets[c]
        self.tm.team_moe_route(self.cfg, xs[step], self.T, d_w["router"], ms[step][M], self.r_idx, self.r_gate, None, self.ws)
        self.torch.cuda.synchronize()
        v = self.r_idx.cpu().numpy()
        return int(np.unique(v[v >= 0]).size)

    def touched(self, M):
        return float(np.mean([self.n_touched(c, 0, M) for c in range(min(self.n_sets, 4))]))

    def bench_step(self, i, M, w8=False):
        """One timed step: one layer call (cfg2/3/5, rotating weight sets) or one pass over the whole stack (cfg4)."""
        if self.wl == "cfg4":
            for c in range(self.n_sets):
                self.layer(c, i % self.steps_per_block, M, w8)
        else:
            self.layer(i % self.n_sets, 0, M, w8)

    def time_steps(self, M, steps, warmup, w8=False):
        torch = self.torch
        for i in range(warmup):
            self.bench_step(i, M, w8)
        torch.cuda.synchronize()
        t_begin = time.perf_counter()
        for i in range(steps):
            self.bench_step(i, M, w8)
        torch.cuda.synchronize()
        return (time.perf_counter() - t_begin) / steps

    def time_ffn(self, M, calls, warmup, w8=False):
        """Duration of the expert FFN kernel inside whole-layer calls: two HIP events per call, recorded by the library on the
        launch stream directly before and after that one kernel (team_moe_layer_args.ffn_begin_event / ffn_end_event).
        Returns (mean, median, min) in seconds."""
        torch = self.torch
        pairs = []
        for i in range(warmup + calls):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(self.stream)                           # (creates the handles; re-recorded by the call below)
            e1.record(self.stream)
            c = i % self.n_sets
            self.layer(c, (i // self.n_sets) % self.steps_per_block, M, w8, events=(e0.cuda_event, e1.cuda_event))
            if i >= warmup:
                pairs.append((e0, e1))
        torch.cuda.synchronize()
        ms = np.array([a.elapsed_time(b) for a, b in pairs])
        return float(ms.mean()) * 1e-3, float(np.median(ms)) * 1e-3, float(ms.min()) * 1e-3

    def chunked_step_times(self, M, chunks=20, per_chunk=20):
        """Median and minimum over groups of back-to-back steps (seconds per step), outside the timed region."""
        torch = self.torch
        times = []
        for c in range(chunks):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(per_chunk):
                self.bench_step(c * per_chunk + i, M)
            torch.cuda.synchronize()
            times.append((time.perf_counter() - t0) / per_chunk)
        return float(np.median(times)), float(np.min(times))

    def sweep_entry(self, M, s_step, ffn, touched, w8=False):
        s_layer = s_step / self.layers_per_step
        s_ffn, s_med, s_min = ffn
        bpe = (3 * self.H * self.I + (2 * self.I + self.H) * 4) if w8 else self.bytes_per_expert
        wbytes = touched * bpe
        flops = 2.0 * self.A * 3 * self.H * self.I
        return {"activated": M, "touched": touched, "ms_per_layer": s_layer * 1e3, "tokens_per_s": self.T / s_step,
                "ffn_ms": s_ffn * 1e3, "ffn_ms_median": s_med * 1e3, "ffn_ms_min": s_min * 1e3, "weight_bytes_per_launch": wbytes,
                "weight_GBps_ffn": wbytes / s_ffn / 1e9, "weight_GBps_layer": wbytes / s_layer / 1e9,
                "frac_of_hbm_peak": wbytes / s_ffn / 1e9 / HBM_PEAK_GBS, "non_ffn_share_of_layer": max(0.0, 1.0 - s_ffn / s_layer),
                "ffn_TFLOPs": flops / s_ffn / 1e12, "mfma_frac": flops / s_ffn / 1e12 / MFMA_BF16_PEAK_TFLOPS}

    # ---- parity of what the timed call produces: set 0, step 0, against the oracle at the layer's bar
    def parity(self, M, threads=0):
        from oracle import c_oracle as orc
        torch, gen = self.torch, self.gen
        xh, w, masks_h, lg = self.host0
        mask = masks_h[M]
        t0 = time.time()
        self.layer(0, 0, M)
        torch.cuda.synchronize()
        y_gpu = self.y.float().cpu().numpy().astype(np.float64)
        d_w, xs, ms = self.sets[0]
        self.tm.team_moe_route(self.cfg, xs[0], self.T, d_w["router"], ms[0][M], self.r_idx, self.r_gate, None, self.ws)
        torch.cuda.synchronize()
        g_idx, g_gate = self.r_idx.cpu().numpy(), self.r_gate.cpu().numpy()
        wf = {n: gen.as_f32(a) for n, a in w.items()}
        xf = gen.as_f32(xh)
        o_y, o_idx, _ = orc.moe_layer(xf, wf["router"], wf["gate"], wf["up"], wf["down"], self.k, 1, mask, threads=threads)
        same = np.array([sorted(g_idx[t].tolist()) == sorted(o_idx[t].tolist()) for t in range(self.T)])
        # tokens whose k-th and (k+1)-th allowed scores are within GAP may select differently: compared with the oracle's expert
        # FFN + combine on the GPU's own selection; every other token must select what the oracle selects
        allowed = np.ones(self.E, bool) if mask is None else mask != 0
        z = np.sort(lg[:, allowed].astype(np.float64), axis=1)[:, ::-1]
        k_eff = min(self.k, z.shape[1])
        safe = np.ones(self.T, bool) if z.shape[1] <= k_eff else (z[:, k_eff - 1] - z[:, k_eff]) > GAP
        indices_ok = bool(same[safe].all())
        ref = o_y.copy()
        if (~same).any():
            rows = np.nonzero(~same)[0]
            o = orc.expert_rows(xf[rows], wf["gate"], wf["up"], wf["down"], g_idx[rows])
            ref[rows] = orc.combine(o, g_gate[rows].astype(np.float64), g_idx[rows])
        num, den = np.abs(y_gpu - ref).max(axis=1), np.abs(ref).max(axis=1)
        row_err = float(np.where(den > 0, num / np.where(den > 0, den, 1.0), np.where(num == 0, 0.0, np.inf)).max())
        rms = float(np.sqrt(np.mean(ref * ref)))
        elem = float((np.abs(y_gpu - ref) / np.maximum(np.abs(ref), 1e-3 * rms)).max()) if rms > 0 else 0.0
        del wf
        return {"checked": f"y of one timed call (weight set 0, M={M}, {self.T} tokens) against the CPU oracle", "row_rel_err": row_err,
                "bar": PARITY_BAR, "elem_err_floor_1e-3_rms": elem, "indices_match_outside_gap_band": indices_ok,
                "tokens_in_gap_band": int((~safe).sum()), "tokens_teacher_forced": int((~same).sum()),
                "pass": bool(row_err <= PARITY_BAR and indices_ok), "seconds": time.time() - t0}

    def free(self):
        self.sets, self.sets_q, self.host0 = [], [], None
        self.torch.cuda.empty_cache()


def stream_ceilings(torch, tm, sizes_mb):
    """Practical ceilings measured in this run, per buffer size: a plain device-to-device copy (read + write bytes over the
    time) and a plain read-only stream (team_moe_internal_stream_read: the expert FFN's kind of load, data discarded)."""
    dev = "cuda:0"
    stream = torch.cuda.current_stream()
    out = []
    big = max(sizes_mb) * 1000 * 1000
    n_rot = 4                                                   # rotate over distinct buffers so that nothing is served by the 256 MB cache
    srcs = [torch.empty(big, dtype=torch.uint8, device=dev).random_(0, 255) for _ in range(n_rot)]
    dst = torch.empty(big, dtype=torch.uint8, device=dev)
    sink = torch.zeros(4096, dtype=torch.int32, device=dev)
    for mb in sizes_mb:
        nbytes = mb * 1000 * 1000 // 16 * 16
        reps = 12
        def timed(fn):
            for i in range(3):
                fn(i)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for i in range(reps):
                fn(i)
            e1.record(stream)
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e-3 / reps
        t_copy = timed(lambda i: dst[:nbytes].copy_(srcs[i % n_rot][:nbytes]))
        t_read = timed(lambda i: tm.internal_stream_read(srcs[i % n_rot], nbytes, sink, 2048))
        out.append({"MB": mb, "copy_GBps_read_plus_write": 2.0 * nbytes / t_copy / 1e9, "read_only_GBps": nbytes / t_read / 1e9,
                    "read_only_us": t_read * 1e6})
    del srcs, dst
    torch.cuda.empty_cache()
    return out


def cpu_baseline(wlo, M, seconds):
    """The oracle, as it stands, on the headline workload (weight set 0) on this machine's host cores: all cores, and one thread."""
    from oracle import c_oracle as orc
    gen = wlo.gen
    xh, w, masks_h, _ = wlo.host0
    wf = {n: gen.as_f32(a) for n, a in w.items()}
    xf = gen.as_f32(xh)
    mask = masks_h[M]
    T, k = wlo.T, wlo.k
    n_all = orc.max_threads()
    orc.moe_layer(xf, wf["router"], wf["gate"], wf["up"], wf["down"], k, 1, mask)          # warm
    n, t_begin = 0, time.perf_counter()
    while time.perf_counter() - t_begin < seconds:
        orc.moe_layer(xf, wf["router"], wf["gate"], wf["up"], wf["down"], k, 1, mask)
        n += 1
    el = time.perf_counter() - t_begin
    t1 = time.perf_counter()
    orc.moe_layer(xf, wf["router"], wf["gate"], wf["up"], wf["down"], k, 1, mask, threads=1)
    el1 = time.perf_counter() - t1
    orc.moe_layer(xf[:1], wf["router"], wf["gate"], wf["up"], wf["down"], k, 1, mask, threads=n_all)   # (thread count back to all cores)
    return {"value": T * n / el / wlo.layers_per_step, "unit": "tokens/s", "cores": n_all, "kind": "oracle",
            "sample": f"{n} single-layer calls of the same workload (weight set 0, M={M}, {T} tokens each) in {el:.1f}s on all cores"
                      + (f"; scaled to the {wlo.layers_per_step}-layer step" if wlo.layers_per_step > 1 else "")
                      + f"; one call on a single thread: {el1:.2f}s",
            "single_thread_value": T / el1 / wlo.layers_per_step, "host_cpu_count": os.cpu_count()}


def workload_description(wl, wlo, M):
    n_sets = wlo.n_sets
    return {
        "cfg2": f"cfg2: one 30B-A3B-shaped MoE layer (H=2048, E=128, top-8, I=768, bf16), block of 32 tokens, activated-expert set "
                f"M={M} (top experts by summed router probability), {n_sets} weight sets rotated",
        "cfg3": f"cfg3: same layer, 4 speculative candidates x 32 tokens = 128 tokens sharing one activated set of {M} experts, "
                f"{n_sets} weight sets rotated",
        "cfg4": f"cfg4: stack of {n_sets} cfg2 layers (MoE FFN only; the configuration has 48, the layers are independent so the per-layer "
                f"figures do not depend on the count), one 32-token block, 16 denoising steps with drifting hidden states, activated set of "
                f"{M} per (layer, step); a step = one pass over the stack",
        "cfg5": f"cfg5: fine-grained layer (H=2048, E=256, top-8, I=512, bf16), 256 tokens, activated set M={M}, {n_sets} weight sets rotated",
    }[wl]


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", choices=["all", "cfg2", "cfg3", "cfg4", "cfg5", "block"], default="all",
                    help="all (default): the cfg2 headline and sweep, then cfg3, cfg4 and cfg5 under 'workloads'; cfgN: that workload alone as the headline")
    ap.add_argument("--copies", type=int, default=0, help="distinct weight sets rotated over (default 4; cfg4: layers of the stack, default 8 of the 48)")
    ap.add_argument("--masks", type=str, default="",
                    help="activated-set sizes of the sweep (the headline size is always measured); e.g. --masks 32 for a profile of the headline only")
    ap.add_argument("--w8", action="store_true",
                    help="time the layer on 8-bit expert weights (E4M3 codes + row scales) instead of bf16 weights (not the headline)")
    ap.add_argument("--block-x", choices=["structured", "drift"], default="structured",
                    help="block workload: hidden states with a component shared by the rows of the block (default), or independent rows")
    ap.add_argument("--tokens", type=int, default=0,
                    help="cfg2 / cfg5 only: another number of tokens per call than the configuration's (a look beyond the listed workloads)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle legs (baseline and parity)")
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
    torch.cuda.set_device(0)
    everything = args.workload == "all"
    wl = "cfg2" if everything else args.workload
    if args.tokens > 0:
        assert wl in ("cfg2", "cfg5") and args.tokens <= 1024, "--tokens: cfg2 / cfg5, at most 1024 tokens per call"
    headline = WORKLOADS[wl][4]
    mask_sizes = tuple(sorted({int(v) for v in args.masks.split(",") if v} | {headline}, reverse=True)) if args.masks else None
    wlo = Workload(wl, args, torch, tm, gen, n_sets=args.copies or None, tokens=args.tokens, mask_sizes=mask_sizes)
    T, H, E, k, I, A = wlo.T, wlo.H, wlo.E, wlo.k, wlo.I, wlo.A
    if args.w8:
        assert wlo.w8_supported(), "8-bit weights need hidden 1024 or 2048 and inter a multiple of 256"

    # ---- headline: exactly `steps` timed steps between synchronisations
    steps, warmup = (max(2, args.steps // 50), max(1, args.warmup // 20)) if wl == "cfg4" else (args.steps, args.warmup)
    sec_per_step = wlo.time_steps(headline, steps, warmup, args.w8)
    sweep = []
    for M in wlo.mask_sizes:
        s_step = sec_per_step if M == headline else wlo.time_steps(M, max(50, steps // 2), max(10, warmup // 2), args.w8)
        ffn = wlo.time_ffn(M, max(50, args.steps // 2), max(10, args.warmup // 2), w8=args.w8)
        e = wlo.sweep_entry(M, s_step, ffn, wlo.touched(M), args.w8)
        sweep.append(e)
        log(f"[bench] {wl} M={M}: layer {e['ms_per_layer'] * 1e3:.1f} us, ffn {e['ffn_ms'] * 1e3:.1f} us, touched {e['touched']:.1f}, "
            f"ffn weight stream {e['weight_GBps_ffn']:.0f} GB/s ({e['frac_of_hbm_peak']:.3f} of peak), {e['ffn_TFLOPs']:.1f} TFLOP/s, "
            f"outside the FFN kernel {100 * e['non_ffn_share_of_layer']:.0f}% of the layer")
    head = next(r for r in sweep if r["activated"] == headline)
    traffic = PMC_TRAFFIC.get((wl, headline)) if not args.w8 and args.tokens == 0 else None
    roofline = {"bound": "hbm", "kernel": "ffn_fused_kernel (the expert FFN of the layer call: gate/up + down GEMMs of the activated experts, one launch)",
                "achieved": head["weight_GBps_ffn"], "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": head["weight_GBps_ffn"] / HBM_PEAK_GBS,
                "traffic": traffic[0] if traffic else None, "traffic_source": traffic[1] if traffic else None,
                "bytes_per_launch": head["weight_bytes_per_launch"], "launch_us": head["ffn_ms"] * 1e3,
                "timed_with": "HIP events recorded by the library on the launch stream directly before and after the kernel, inside team_moe_layer_forward_ex"}

    # ---- the same layer with the activated set decided on the device (Algorithm 1: two-round routing from token classes)
    two_round = None
    if wl != "cfg4" and not args.masks and not args.w8:
        n_first = max(1, T // 8)
        cls = [torch.from_numpy(gen.token_classes(T, n_first, seed=c)).to(wlo.dev) for c in range(wlo.n_sets)]
        d_nact = torch.zeros((1,), dtype=torch.int32, device=wlo.dev)
        d_mask = torch.zeros((E,), dtype=torch.uint8, device=wlo.dev)

        def layer2(i):
            d_w, xs, ms = wlo.sets[i % wlo.n_sets]
            tm.team_moe_layer_forward_two_round(wlo.cfg, xs[0], T, d_w["router"], d_w["gate"], d_w["up"], d_w["down"], cls[i % wlo.n_sets],
                                                d_mask, d_nact, wlo.y, wlo.ws)

        n_act = []
        for c in range(wlo.n_sets):
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
    if wl == "cfg2" and wlo.w8_supported() and not args.masks and not args.w8 and args.tokens == 0:
        s8 = wlo.time_steps(headline, max(50, steps // 2), 10, w8=True)
        f8 = wlo.time_ffn(headline, max(50, args.steps // 2), 10, w8=True)
        e8 = wlo.sweep_entry(headline, s8, f8, head["touched"], w8=True)
        w8 = {"weights": "E4M3 codes + one float scale per row", "activated": headline, "ms_per_layer": e8["ms_per_layer"],
              "tokens_per_s": e8["tokens_per_s"], "ffn_ms": e8["ffn_ms"], "weight_bytes_per_launch": e8["weight_bytes_per_launch"],
              "weight_GBps_ffn": e8["weight_GBps_ffn"], "frac_of_hbm_peak": e8["frac_of_hbm_peak"]}
        log(f"[bench] {wl} M={headline} on 8-bit weights: layer {s8 * 1e6:.1f} us, ffn {f8[0] * 1e6:.1f} us, weight stream {e8['weight_GBps_ffn']:.0f} GB/s")

    # ---- candidate branches with repeated rows (Section "Aligned Token Candidates in SEH"): the same layer over 4 x 32 rows of
    #      which 34 are distinct, computed row by row and with every distinct row computed once
    branches = None
    if wl == "cfg3" and not args.masks:
        from oracle import c_oracle as orc
        bx, bm = [], []
        for c in range(wlo.n_sets):
            xh = gen.make_x(wlo.shape, seed=0, layer=0, step=c, kind="branches")
            bx.append(wlo.dev_t(xh))
            lg = orc.router_logits(gen.as_f32(xh), wlo.sets[c][0]["router"].float().cpu().numpy())
            bm.append(torch.from_numpy(gen.activated_set_by_summed_probability(lg, headline)).to(wlo.dev))
        d_rep = torch.zeros((T,), dtype=torch.int32, device=wlo.dev)
        d_nu = torch.zeros((1,), dtype=torch.int32, device=wlo.dev)

        def plain(i):
            d_w = wlo.sets[i % wlo.n_sets][0]
            tm.team_moe_layer_forward(wlo.cfg, bx[i % wlo.n_sets], T, d_w["router"], d_w["gate"], d_w["up"], d_w["down"], bm[i % wlo.n_sets], wlo.y, wlo.ws)

        def unique(i):
            d_w = wlo.sets[i % wlo.n_sets][0]
            tm.team_moe_layer_forward_unique_rows(wlo.cfg, bx[i % wlo.n_sets], T, d_w["router"], d_w["gate"], d_w["up"], d_w["down"],
                                                  bm[i % wlo.n_sets], wlo.y, d_rep, d_nu, wlo.ws)

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

    med_min = None
    if wl != "cfg4":
        med_min = wlo.chunked_step_times(headline)

    # ---- parity of the timed call and the CPU baseline (the oracle on this machine's host cores)
    parity, cpu = None, None
    if not args.no_cpu:
        parity = wlo.parity(headline)
        log(f"[bench] {wl} M={headline} parity against the oracle: row error {parity['row_rel_err']:.2e} (bar {PARITY_BAR}), pass={parity['pass']}")
        cpu = cpu_baseline(wlo, headline, args.cpu_seconds)
    desc = workload_description(wl, wlo, headline)
    if args.tokens > 0:
        desc = f"{wl} shape at {T} tokens per call instead of the configuration's (not a listed workload): " + desc
    touched_head, layers_per_step = head["touched"], wlo.layers_per_step

    # ---- the other listed workloads, each measured the same way (layer time, FFN kernel by events, parity of one timed call)
    workloads = None
    if everything:
        workloads = []
        wlo.free()
        for other in ("cfg3", "cfg4", "cfg5"):
            o = Workload(other, args, torch, tm, gen)
            for M in o.mask_sizes:
                o_steps = max(4, args.steps // 50) if other == "cfg4" else max(100, args.steps // 2)
                s_step = o.time_steps(M, o_steps, max(2, o_steps // 10))
                ffn = o.time_ffn(M, 100, 10)
                e = o.sweep_entry(M, s_step, ffn, o.touched(M))
                e["workload"] = workload_description(other, o, M)
                e["name"] = f"{other}_M{M}"
                e["tokens"] = o.T
                if other == "cfg4":
                    e["ms_per_step_over_this_stack"] = s_step * 1e3
                    e["ms_per_step_48_layers"] = e["ms_per_layer"] * 48
                    e["ms_per_block_16_steps_48_layers"] = e["ms_per_layer"] * 48 * 16
                e["parity"] = None if args.no_cpu else o.parity(M)
                workloads.append(e)
                log(f"[bench] {other} M={M}: layer {e['ms_per_layer'] * 1e3:.1f} us, ffn {e['ffn_ms'] * 1e3:.1f} us, touched {e['touched']:.1f}, "
                    f"{e['weight_GBps_ffn']:.0f} GB/s ({e['frac_of_hbm_peak']:.3f} of peak), {e['ffn_TFLOPs']:.1f} TFLOP/s"
                    + ("" if args.no_cpu else f", parity row error {e['parity']['row_rel_err']:.2e} pass={e['parity']['pass']}"))
            o.free()
            del o
    else:
        wlo.free()

    # ---- context: practical ceilings of this device at the sizes the expert FFN streams, measured in this run
    ceilings = stream_ceilings(torch, tm, (151, 302, 604, 1208))
    log("[bench] ceilings: " + "; ".join(f"{c['MB']} MB: copy {c['copy_GBps_read_plus_write']:.0f} GB/s, read-only {c['read_only_GBps']:.0f} GB/s" for c in ceilings))

    out = {"metric": "moe_layer_tokens_per_s", "value": T / sec_per_step, "unit": "tokens/s", "n_gpus": 1, "steps": steps,
           "warmup": warmup, "ms_per_step": sec_per_step * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "bf16", "data": "synthetic" + (" (expert weights stored as E4M3 codes with row scales)" if args.w8 else ""),
           "config": {"workload": desc, "tokens": T, "activated": headline, "touched": touched_head, "layers_per_step": layers_per_step},
           "roofline": roofline, "cpu_baseline": cpu, "parity": parity, "sweep": sweep, "workloads": workloads, "two_round": two_round,
           "branches": branches, "w8": w8, "ceilings": ceilings,
           "device_copy_GBps": next(c["copy_GBps_read_plus_write"] for c in ceilings if c["MB"] == 1208)}
    if wl == "cfg4":
        out["ms_per_block_16_steps"] = sec_per_step * 1e3 * 16
    else:
        out["ms_per_step_median"], out["ms_per_step_min"] = med_min[0] * 1e3, med_min[1] * 1e3
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
