#!/usr/bin/env python3
"""Benchmark of the single-GPU FlexMoE MoE-layer hot path on one MI355X.

A step is one pass of the whole hot path over one synthetic batch:
  forward  = gate_topk -> route -> permute -> expert_ffn_fwd -> combine
  backward = permute(dY, gate weights) -> expert_ffn_bwd -> combine      (training configs)
all through the C ABI of libflexmoe.so, inputs resident in HBM before the timed region.

The default workload is the GPT-XL-like layer (the largest single-GPU configuration: 65536 tokens,
d = 2048, f = 8192, 64 experts, top-2, forward + backward, hot set drifting every 10 steps).

Prints one JSON line: whole-job tokens/s, the roofline of the dominant kernels (the grouped-GEMM
expert FFN of the whole step, MFMA-bound; HIP events around its calls inside the timed steps) with
per-stage figures, a compact table of the other configurations, and the CPU oracle timed on the
host cores as a reported baseline.
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

MFMA_BF16_PEAK_TFLOPS = 2500.0     # MI355X dense bf16
FP32_VECTOR_PEAK_TFLOPS = 157.3
HBM_PEAK_GBS = 8000.0



def measured_ffn_traffic_bytes(name):
    """HBM bytes that the grouped-GEMM launches of one step move (flexmoe_expert_ffn_fwd + flexmoe_expert_ffn_bwd),
    from two rocprofv3 --pmc runs of this script (FETCH_SIZE, then WRITE_SIZE), each scaled by what the same counter
    reads for a plain 1 GiB device copy.  Read from the committed summary profiles/ffn_<workload>_hbm_traffic.txt
    (line `TRAFFIC_BYTES_PER_STEP <bytes>`); None when no summary exists for the workload."""
    path = os.path.join(ROOT, "profiles", f"ffn_{name}_hbm_traffic.txt")
    try:
        with open(path) as fh:
            for ln in fh:
                if ln.startswith("TRAFFIC_BYTES_PER_STEP"):
                    return float(ln.split()[1])
    except OSError:
        pass
    return None


WORKLOAD_TEXT = {
    "tiny": "configs[0] tiny fp32 MoE layer, forward",
    "bert": "configs[1] BERT-base-like MoE layer bf16, forward, 8192 tokens, d=768, f=3072, E=16, k=2, V=18",
    "gpt_m": "configs[2] GPT-medium-like MoE layer bf16, forward+backward, 16384 tokens, d=1024, f=4096, E=32, k=2, V=48",
    "swin": "configs[3] Swin-like MoE layer bf16, forward+backward, 32768 tokens, d=512, f=2048, E=32, k=1, V=40",
    "gpt_xl": "configs[4] GPT-XL-like MoE layer bf16, forward+backward, 65536 tokens, d=2048, f=8192, E=64, k=2, V=96, hot set drifts every 10 steps",
}


def stage_work(cfg):
    """Algorithmic bytes / flops of each stage of one step (what the method must move or compute)."""
    from paper_2304_03946_amd import workloads as W
    s = 2 if cfg.dtype == W.DT_BF16 else 4
    N, d, f, E, k, A = cfg.N, cfg.d, cfg.f, cfg.E, cfg.k, cfg.A
    work = {
        "gate": ("hbm", N * d * s + d * E * s + 8 * A),
        "route": ("hbm", 12 * A),
        "permute": ("hbm", N * d * s + A * d * s + 4 * A),
        "ffn_fwd": ("mfma", 4 * A * d * f),
        "combine": ("hbm", A * d * s + N * d * s + 8 * A),
    }
    if cfg.backward:
        work["bwd_permute"] = ("hbm", N * d * s + A * d * s + 8 * A)
        work["ffn_bwd"] = ("mfma", 8 * A * d * f)
        work["bwd_combine"] = ("hbm", A * d * s + N * d * s + 4 * A)
    return work


class Runner:
    keep_h = True      # training layers: the forward pass keeps act(Hpre) for the backward pass (--recompute-h turns it off)

    def __init__(self, name, seed=None, fused=False):
        import torch
        from paper_2304_03946_amd import binding, layer, workloads as W
        self.torch, self.W, self.layer_mod = torch, W, layer
        binding.load_library()
        self.cfg = cfg = W.CONFIGS[name]
        self.name = name
        self.inp = inp = W.make_layer_inputs(cfg, seed=seed)
        up = layer.to_device
        self.x, self.w1, self.w2, self.dy = up(inp.x), up(inp.w1), up(inp.w2), up(inp.dy)
        self.wg_by_drift = {0: up(inp.wg)}
        self.L = layer.MoELayer(cfg.N, cfg.d, cfg.f, cfg.E, cfg.k, cfg.V, cfg.dtype, cfg.act, cfg.backward, keep_h=Runner.keep_h)
        self.iter = 0
        self.drifting = name == "gpt_xl"
        # without a backward pass nothing reads Xp again: fold the permutation into the expert GEMM
        self.fused = fused and not cfg.backward and self.L.gather_supported()
        self.keep_hpre = True
        # placement: the benchmark's table for the BERT-like layer; otherwise the greedy
        # capacity rule on the loads observed on a first (untimed) pass
        self.rep = W.config_placement(cfg)
        if cfg.V != cfg.E and name != "bert":
            self.L.gate(self.x, self.wg_by_drift[0])
            self.L.route(*self.rep)
            torch.cuda.synchronize()
            self.rep = W.placement_from_loads(self.L.expert_count.cpu().numpy(), cfg.V, cfg.max_rep)

    def prepare_drifts(self, total_steps):
        if not self.drifting:
            return
        for j in range(total_steps // 10 + 1):
            if j not in self.wg_by_drift:
                wg, _ = self.W.make_gate_weights(self.cfg, self.inp.seed, drift=j)
                self.wg_by_drift[j] = self.layer_mod.to_device(wg)

    def step(self, timers=None, ffn_events=None):
        """One pass of the hot path.  `timers`: events after every stage (breakdown pass); `ffn_events`: a list
        that receives (start, end) event pairs around the two grouped-GEMM calls only (timed region)."""
        L, cfg = self.L, self.cfg
        from paper_2304_03946_amd import binding as B
        j = self.iter // 10 if self.drifting else 0
        if self.drifting and self.iter % 10 == 1 and self.iter > 1:
            # the hot set moved on the previous step: new table from the loads that step observed
            # (the read-back and the table build are inside the timed region)
            self.rep = self.W.placement_from_loads(L.expert_count.cpu().numpy(), cfg.V, cfg.max_rep)
        wg = self.wg_by_drift[j]
        rec = timers.record if timers else (lambda name: None)
        rec(None)
        L.gate(self.x, wg); rec("gate")
        L.route(*self.rep); rec("route")
        if self.fused:
            # forward-only layer: the layout transformation rides on GEMM1's row loads (no Xp)
            B.flexmoe_expert_ffn_fwd_gather(self.x, L.src, cfg.k, L.vexpert_off, L.vexpert_owner, self.w1, None,
                                            self.w2, None, cfg.act, L.hpre if self.keep_hpre else None, L.yp,
                                            L.ws); rec("ffn_fwd")
        else:
            B.flexmoe_permute(self.x, L.src, None, cfg.k, L.xp); rec("permute")
            e0 = self._event(ffn_events)
            B.flexmoe_expert_ffn_fwd(L.xp, L.vexpert_off, L.vexpert_owner, self.w1, None, self.w2, None, cfg.act,
                                     L.hpre, L.yp, L.ws, h=L.h); rec("ffn_fwd")      # training layers keep act(Hpre) for the backward pass
            self._event(ffn_events, e0, "fwd")
        B.flexmoe_combine(L.yp, L.dest, L.topk_w, cfg.k, L.y); rec("combine")
        if cfg.backward:
            B.flexmoe_permute(self.dy, L.src, L.topk_w, cfg.k, L.dyp); rec("bwd_permute")
            e0 = self._event(ffn_events)
            B.flexmoe_expert_ffn_bwd(L.dyp, L.xp, L.hpre, self.w1, self.w2, L.vexpert_off, L.vexpert_owner, cfg.act,
                                     L.dxp, L.dw1, L.dw2, L.ws, h=L.h); rec("ffn_bwd")
            self._event(ffn_events, e0, "bwd")
            B.flexmoe_combine(L.dxp, L.dest, None, cfg.k, L.dx); rec("bwd_combine")
        self.iter += 1

    def _event(self, sink, start=None, tag=None):
        """HIP event on the stream the kernels are launched on (torch's current stream)."""
        if sink is None:
            return None
        ev = self.torch.cuda.Event(enable_timing=True)
        ev.record()
        if start is not None:
            sink.append((tag, start, ev))
        return ev


class StageTimers:
    """HIP events on the stream the kernels are launched on (torch's current stream)."""

    def __init__(self, torch):
        self.torch = torch
        self.pairs = {}
        self.last = None

    def record(self, name):
        ev = self.torch.cuda.Event(enable_timing=True)
        ev.record()
        if name is not None:
            self.pairs.setdefault(name, []).append((self.last, ev))
        self.last = ev

    def median_ms(self):
        """Median interval per stage over the steps (an interval also holds the idle time of the stream when
        the host falls behind between two launches; the median is not moved by the few steps where it does)."""
        return {n: median([a.elapsed_time(b) for a, b in p]) for n, p in self.pairs.items()}


def median(values):
    t = sorted(values)
    return 0.5 * (t[(len(t) - 1) // 2] + t[len(t) // 2])


def run_workload(name, steps, warmup, with_stages=True, fused=False, variants=True):
    import torch
    r = Runner(name, fused=fused)
    cfg = r.cfg
    r.prepare_drifts(warmup + steps * 2 + 2)
    for _ in range(warmup):
        r.step()
    torch.cuda.synchronize()
    ffn_events = []
    t0 = time.perf_counter()
    for _ in range(steps):
        r.step(ffn_events=ffn_events)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / steps * 1e3
    out = dict(tokens_per_s=cfg.N / (dt / steps), ms_per_step=ms_per_step, fused=r.fused)
    # the grouped-GEMM calls of the timed steps themselves: per-step duration = forward call + backward call
    per_call = {}
    for tag, a, b in ffn_events:
        per_call.setdefault(tag, []).append(a.elapsed_time(b))
    if per_call:
        per_step = [sum(v) for v in zip(*per_call.values())]
        out["ffn_timed"] = dict(mean_ms=sum(per_step) / len(per_step), median_ms=median(per_step),
                                calls={t: round(sum(v) / len(v), 4) for t, v in per_call.items()})
    if variants and not r.fused and not cfg.backward and r.L.gather_supported():
        # the same forward pass with the permutation folded into the first expert GEMM (no Xp written):
        # reported beside the step, which keeps every stage as a call of its own
        r.fused = True
        for _ in range(warmup):
            r.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            r.step()
        torch.cuda.synchronize()
        dtf = time.perf_counter() - t0
        out["fused_permute"] = dict(ms_per_step=round(dtf / steps * 1e3, 4), tokens_per_s=round(cfg.N / (dtf / steps), 1),
                                    call="flexmoe_expert_ffn_fwd_gather replaces flexmoe_permute + flexmoe_expert_ffn_fwd")
        # and the inference form of that call: hpre = NULL, the pre-activations (kept for a backward pass) are not stored
        r.keep_hpre = False
        for _ in range(warmup):
            r.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            r.step()
        torch.cuda.synchronize()
        dti = time.perf_counter() - t0
        out["fused_permute"]["without_stored_preactivations"] = dict(ms_per_step=round(dti / steps * 1e3, 4),
                                                                     tokens_per_s=round(cfg.N / (dti / steps), 1))
        r.keep_hpre = True
        r.fused = False
    if with_stages:
        timers = StageTimers(torch)
        for _ in range(steps):
            r.step(timers)
        torch.cuda.synchronize()
        stage_ms = timers.median_ms()
        work = stage_work(cfg)
        stages = {}
        for st, ms in stage_ms.items():
            bound, amount = work[st]
            if bound == "mfma":
                peak = MFMA_BF16_PEAK_TFLOPS if cfg.dtype == r.W.DT_BF16 else FP32_VECTOR_PEAK_TFLOPS
                ach = amount / (ms * 1e-3) / 1e12
                stages[st] = dict(ms=round(ms, 4), bound="mfma" if cfg.dtype == r.W.DT_BF16 else "alu",
                                  achieved=round(ach, 2), unit="TFLOP/s", frac=round(ach / peak, 4))
            else:
                ach = amount / (ms * 1e-3) / 1e9
                stages[st] = dict(ms=round(ms, 4), bound="hbm", achieved=round(ach, 1), unit="GB/s",
                                  frac=round(ach / HBM_PEAK_GBS, 4))
        out["stages"] = stages
        if cfg.backward:
            out["trainable_layer_extras"] = time_extras(r, steps)
        out["token_cost_ns"] = r.L.profile_token_cost(r.w1, r.w2)      # Eq. 7: T_C per token from profiling
        counts = r.L.expert_count.cpu().numpy()
        vc = r.L.vexpert_count.cpu().numpy()
        out["loads"] = dict(hottest_expert_share=round(float(counts.max()) / cfg.A, 4),
                            top10_share=round(float(sum(sorted(counts.tolist(), reverse=True)[:10])) / cfg.A, 4),
                            max_vexpert=int(vc.max()), mean_vexpert=round(float(vc.mean()), 1))
    return r, out


def copy_ceiling_gbs(nbytes=1 << 28, reps=20):
    """Read + write rate of a plain device-to-device copy of `nbytes` (the practical ceiling the
    HBM-bound stages are held against, beside the 8 TB/s peak)."""
    import torch
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    return round(2 * nbytes * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)


def read_ceiling_gbs(nbytes=1 << 28, reps=20):
    """Rate of a read-only pass over `nbytes` (a sum reduction): what a stage that reads far more than it
    writes can be held against, beside the copy ceiling."""
    import torch
    src = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda").fill_(1.0)
    for _ in range(3):
        src.sum()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        src.sum()
    e1.record()
    torch.cuda.synchronize()
    return round(nbytes * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)


def dense_gemm_ceiling_tflops(name, reps=10):
    """What the vendor library reaches on this machine for the layer's two forward products taken as
    plain dense GEMMs (all A rows against one expert's weights, no buckets, no fused epilogue):
    torch.matmul in bf16.  A practical ceiling beside the 2.5 PFLOP/s peak, not part of the path."""
    import torch
    from paper_2304_03946_amd import workloads as W
    cfg = W.CONFIGS[name]
    if cfg.dtype != W.DT_BF16:
        return None
    out = {}
    for tag, (m, k, n) in {"gemm1": (cfg.A, cfg.d, cfg.f), "gemm2": (cfg.A, cfg.f, cfg.d)}.items():
        a = torch.randn((m, k), device="cuda", dtype=torch.float32).mul_(0.5).to(torch.bfloat16)
        b = torch.randn((k, n), device="cuda", dtype=torch.float32).mul_(0.02).to(torch.bfloat16)
        c = torch.empty((m, n), device="cuda", dtype=torch.bfloat16)
        for _ in range(3):
            torch.matmul(a, b, out=c)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            torch.matmul(a, b, out=c)
        e1.record()
        torch.cuda.synchronize()
        out[tag] = round(2.0 * m * k * n * reps / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)
        del a, b, c
    return out


def time_extras(r, steps):
    """The gate-path backward and the bias gradients (what a trainable layer needs beyond the hot
    path), timed on their own after a step has left its state in the layer's buffers; not part of
    ms_per_step."""
    import torch
    from paper_2304_03946_amd import binding as B
    L, cfg = r.L, r.cfg
    s = 2 if cfg.dtype == r.W.DT_BF16 else 4
    wg = r.wg_by_drift[0]
    tdt = L.dx.dtype
    db1 = torch.empty((cfg.E, cfg.f), dtype=tdt, device="cuda")
    db2 = torch.empty((cfg.E, cfg.d), dtype=tdt, device="cuda")
    dl = torch.empty((cfg.N, cfg.k), dtype=torch.float32, device="cuda")
    dwg = torch.empty((cfg.d, cfg.E), dtype=tdt, device="cuda")
    calls = {
        "bias_grads": (lambda: B.flexmoe_expert_bias_grads(L.dyp, L.vexpert_off, L.vexpert_owner, cfg.f, cfg.E, db1,
                                                           db2, L.ws),
                       cfg.A * (cfg.f + cfg.d) * s),
        "gate_bwd": (lambda: B.flexmoe_gate_bwd(wg, L.topk_idx, L.topk_w, r.dy, L.yp, L.xp, L.dest, L.src,
                                                L.vexpert_off, L.vexpert_owner, dl, L.dx, dwg, L.ws),
                     (3 * cfg.N + 2 * cfg.A) * cfg.d * s),
    }
    out = {}
    for name, (fn, nbytes) in calls.items():
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / steps
        out[name] = dict(ms=round(ms, 4), bound="hbm", achieved=round(nbytes / (ms * 1e-3) / 1e9, 1), unit="GB/s",
                         frac=round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4))
    if L.top1_supported():
        # top-1 layer, forward only: the staged expert path (permute, FFN, combine) against the one call that
        # gathers on load and scatters on store (flexmoe_expert_ffn_fwd_top1); gate and route are the same
        def staged():
            B.flexmoe_permute(r.x, L.src, None, cfg.k, L.xp)
            B.flexmoe_expert_ffn_fwd(L.xp, L.vexpert_off, L.vexpert_owner, r.w1, None, r.w2, None, cfg.act, L.hpre,
                                     L.yp, L.ws)
            B.flexmoe_combine(L.yp, L.dest, L.topk_w, cfg.k, L.y)

        def fused():
            B.flexmoe_expert_ffn_fwd_top1(r.x, L.src, L.vexpert_off, L.vexpert_owner, r.w1, None, r.w2, None, cfg.act,
                                          L.hpre, L.y, L.ws)
        for name, fn in (("forward_expert_path_staged", staged), ("forward_expert_path_top1_call", fused)):
            fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(steps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / steps
            flops = 4.0 * cfg.A * cfg.d * cfg.f
            out[name] = dict(ms=round(ms, 4), bound="mfma", achieved=round(flops / (ms * 1e-3) / 1e12, 1), unit="TFLOP/s",
                             frac=round(flops / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4))
    return out


def scheduler_pass(name, G=64, S=4, reps=5, token_cost=1):
    """Host-side scheduler (Alg. 1: balance ratio, Policy Maker, Migrate) timed on an emulated cluster of the
    paper's size: G GPUs with S vExpert slots each, every expert owning a contiguous block of slots (the
    static expert-parallel placement), loads = G batches with the workload's expert skew."""
    import numpy as np
    from paper_2304_03946_amd import scheduler as sch
    from paper_2304_03946_amd import workloads as W
    cfg = W.CONFIGS[name]
    V = G * S
    owner = (np.arange(V, dtype=np.int64) * cfg.E // V).astype(np.int32)
    tokens = np.floor(G * W.prior_loads(cfg)).astype(np.int64)
    best = None
    for _ in range(reps):
        t0 = time.perf_counter()
        ops, new_owner, before, after = sch.flexmoe_schedule(tokens, owner, G, token_cost, 1.0, 4 * V)
        dt = time.perf_counter() - t0
        best = dt if best is None else min(best, dt)
    return dict(cluster=f"{G} GPUs x {S} vExpert slots, {cfg.E} experts", token_cost_ns=int(token_cost),
                token_cost_source="HIP-event time of the expert FFN calls per routed token (MoELayer.profile_token_cost)",
                primitives=int(len(ops)),
                balance_ratio_before=round(before, 4), balance_ratio_after=round(after, 4),
                us_per_pass=round(best * 1e6, 1))


def cpu_baseline(name):
    """The CPU oracle as it stands, timed on the host cores on a bounded sample of the workload."""
    import numpy as np
    from threadpoolctl import threadpool_info
    from oracle import flexmoe_oracle as O
    from paper_2304_03946_amd import workloads as W
    cfg = W.CONFIGS[name]
    # bound the sample to about 0.15 TFLOP of fp64 work (a few seconds to tens of seconds on host cores)
    per_token = (4 + (8 if cfg.backward else 0)) * cfg.k * cfg.d * cfg.f
    n = int(min(cfg.N, max(256, 0.15e12 // per_token)))
    sub = W.scaled(cfg, N=n)
    w = W.make_layer_inputs(sub)      # same shapes and distributions as the workload, fewer tokens
    rep = W.config_placement(cfg) if cfg.V == cfg.E or name == "bert" else W.placement_from_loads(W.prior_loads(cfg), cfg.V, cfg.max_rep)
    x, wg = W.decode(w.x), W.decode(w.wg)
    best = None
    reps = 3 if per_token * n < 0.1e12 else 1
    for _ in range(reps):
        t0 = time.perf_counter()
        fwd = O.staged_forward(x, wg, w.w1, None, w.w2, None, cfg.k, cfg.act, rep[0], rep[1])
        if cfg.backward:
            O.staged_backward(fwd, W.decode(w.dy), w.w1, w.w2, cfg.k, cfg.act)
        dt = time.perf_counter() - t0
        best = dt if best is None else min(best, dt)
    threads = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    return dict(value=round(n / best, 1), unit="tokens/s", cores=int(threads), kind="oracle (numpy fp64, threaded BLAS)",
                sample=f"{n} of {cfg.N} tokens of the same layer ({'forward+backward' if cfg.backward else 'forward'}), "
                       f"best of {reps}, {best:.2f} s")


FFN_KERNELS = {
    True: "flexmoe_expert_ffn_fwd (rows_gemm_persist_bf16 x2: GEMM1 + Hpre/GELU epilogue, GEMM2) + flexmoe_expert_ffn_bwd "
          "(rows_gemm_persist_bf16: dH + GELU' epilogue, dXp; wgrad_gemm_persist_bf16: dW2, dW1)",
    False: "flexmoe_expert_ffn_fwd (two grouped-GEMM launches: rows_gemm_persist_bf16 x2)",
}


def compact_row(name, steps, warmup):
    """One short run of another configuration for the compact table of the default line."""
    import torch
    r, o = run_workload(name, steps, warmup, with_stages=False, variants=False)
    cfg = r.cfg
    flops = (12 if cfg.backward else 4) * cfg.A * cfg.d * cfg.f
    row = dict(passes="forward+backward" if cfg.backward else "forward", tokens_per_s=round(o["tokens_per_s"], 1),
               ms_per_step=round(o["ms_per_step"], 4))
    if "ffn_timed" in o:
        peak = MFMA_BF16_PEAK_TFLOPS if cfg.dtype == r.W.DT_BF16 else FP32_VECTOR_PEAK_TFLOPS
        row["ffn_ms"] = round(o["ffn_timed"]["mean_ms"], 4)
        row["ffn_frac_of_peak"] = round(flops / (o["ffn_timed"]["mean_ms"] * 1e-3) / 1e12 / peak, 4)
    del r
    torch.cuda.empty_cache()
    return row


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="gpt_xl", choices=list(WORKLOAD_TEXT))
    ap.add_argument("--all-workloads", action="store_true", help="also time the other configurations stage by stage (extra JSON field)")
    ap.add_argument("--no-others", action="store_true", help="leave out the compact table of the other configurations")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--fused", action="store_true",
                    help="forward-only workloads: time the step with flexmoe_expert_ffn_fwd_gather instead of "
                         "flexmoe_permute + flexmoe_expert_ffn_fwd")
    ap.add_argument("--no-variants", action="store_true",
                    help="do not also time the forward variants reported beside the step (fused permutation, no stored "
                         "pre-activations): profiles then hold the step's own launches only")
    ap.add_argument("--no-stages", action="store_true", help="skip the per-stage breakdown pass (profiled runs: the "
                    "kernel trace then holds warm-up + timed steps only)")
    ap.add_argument("--recompute-h", action="store_true",
                    help="training layers: do not keep act(Hpre) from the forward pass; the backward pass computes and "
                         "stores it again (saves A*f elements of activation memory per layer, costs time)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run a plain 1 GiB device copy (calibrates FETCH_SIZE / WRITE_SIZE under rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs the MoE-layer hot path on ONE GPU; --gpus N with N > 1 is not supported "
                 "(no collectives, no sharding in this library).")
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback.")
    from paper_2304_03946_amd import workloads as W
    name = args.workload
    big = name == "gpt_xl"
    steps = args.steps if args.steps is not None else (30 if big else 200)
    warmup = args.warmup if args.warmup is not None else (3 if big else 20)

    Runner.keep_h = not args.recompute_h
    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    r, res = run_workload(name, steps, warmup, with_stages=not args.no_stages, fused=args.fused,
                          variants=not args.no_variants)
    cfg = r.cfg
    bf16 = cfg.dtype == W.DT_BF16
    peak = MFMA_BF16_PEAK_TFLOPS if bf16 else FP32_VECTOR_PEAK_TFLOPS
    flops = (12 if cfg.backward else 4) * cfg.A * cfg.d * cfg.f      # 4 A d f forward, 8 A d f backward
    ffn = res.get("ffn_timed")
    if ffn is None:      # --fused: the gathered forward call is timed by the stage pass only
        ffn = dict(mean_ms=res["stages"]["ffn_fwd"]["ms"], median_ms=res["stages"]["ffn_fwd"]["ms"], calls={})
    achieved = flops / (ffn["mean_ms"] * 1e-3) / 1e12
    passes = "forward+backward" if cfg.backward else "forward"
    line = {
        "metric": f"MoE-layer tokens/sec ({'fwd+bwd' if cfg.backward else 'fwd'}) on 1 MI355X; grouped-GEMM MFMA util % of peak",
        "value": round(res["tokens_per_s"], 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": round(res["ms_per_step"], 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32",
        "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT[name], "passes": passes,
                   "tokens": cfg.N, "d_model": cfg.d, "d_ff": cfg.f, "experts": cfg.E, "top_k": cfg.k,
                   "vexperts": cfg.V, **({"loads": res["loads"]} if "loads" in res else {}),
                   "permute": "folded into the first expert GEMM (flexmoe_expert_ffn_fwd_gather)" if res["fused"]
                              else "flexmoe_permute", **({"fused_permute": res["fused_permute"]} if "fused_permute" in res else {})},
        "roofline": {"kernel": "flexmoe_expert_ffn_fwd_gather (two grouped-GEMM launches)" if res["fused"] else FFN_KERNELS[cfg.backward],
                     "bound": "mfma" if bf16 else "alu", "achieved": round(achieved, 2), "peak": peak,
                     "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
                     "traffic": None if res["fused"] else measured_ffn_traffic_bytes(name),
                     "launch_ms": round(ffn["mean_ms"], 4), "launch_ms_median": round(ffn["median_ms"], 4),
                     "launch_ms_by_call": ffn["calls"], "algorithmic_flops": flops,
                     "timing": "HIP events around the grouped-GEMM calls of every timed step, on the stream the kernels "
                               "run on; launch_ms = mean over the timed steps of (forward call + backward call), no step left out",
                     **({"stages": res["stages"], "stage_timing": "median over a separate pass of the same steps with an "
                         "event after every call"} if "stages" in res else {})},
    }
    if "trainable_layer_extras" in res:
        line["trainable_layer_extras"] = res["trainable_layer_extras"]
    if not args.no_others and not args.all_workloads:
        del r
        torch.cuda.empty_cache()
        r = None
        line["other_workloads"] = {w: compact_row(w, 20 if w == "gpt_xl" else 100, 3 if w == "gpt_xl" else 10)
                                   for w in ("bert", "gpt_m", "swin", "gpt_xl", "tiny") if w != name}
    if args.all_workloads:
        line["copy_ceiling_GBs"] = {"256MiB": copy_ceiling_gbs(1 << 28), "32MiB": copy_ceiling_gbs(1 << 25, 100)}
        line["read_ceiling_GBs"] = {"256MiB": read_ceiling_gbs(1 << 28)}
        torch.cuda.empty_cache()
        line["dense_gemm_ceiling_TFLOPs"] = {w: dense_gemm_ceiling_tflops(w) for w in ("bert", "gpt_m", "swin", "gpt_xl")}
        others = {}
        for other in ("gpt_m", "swin", "gpt_xl", "bert", "tiny"):
            if other == name:
                continue
            del r
            torch.cuda.empty_cache()
            ob = other == "gpt_xl"
            r, o = run_workload(other, 20 if ob else 100, 3 if ob else 10, fused=args.fused)
            others[other] = dict(tokens_per_s=round(o["tokens_per_s"], 1), ms_per_step=round(o["ms_per_step"], 4),
                                 stages=o["stages"], loads=o["loads"])
            if "trainable_layer_extras" in o:
                others[other]["trainable_layer_extras"] = o["trainable_layer_extras"]
        line["all_workloads"] = others
    line["scheduler"] = scheduler_pass(name, token_cost=res.get("token_cost_ns", 1))
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(name)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
