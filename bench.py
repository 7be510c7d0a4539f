#!/usr/bin/env python3
"""Benchmark of the AMS-KV hot path on one MI355X.

One "step" is one whole pass of the hot path over one image batch of synthetic input, already
resident in HBM: for every scale s and every layer l, amskv_append_scale (policy -> kept set,
eviction, slot assignment) then amskv_attend (which, with fuse_append, also writes the scale it
streams into its cache slot); at the probe scale, amskv_interscale_similarity for every layer;
bytes-held accounting at the end.  Defaults: PLANNED layout, borrow_unretained, fuse_append (the
configuration with the least HBM traffic); --layout compact --no-borrow --no-fuse gives the plain
evict + compact + copy path, whose kernels are also timed once per run ("standalone_append").
Default workload: VAR-d30 shape (30 layers, 30 heads x 64, ten scales = 680 tokens), bf16, batch 256,
cache-demanding layers chosen by the similarity call (mean cosine < 0.5 -> keep all scales), the rest
{0,1} + window 2.

Prints ONE JSON line.  `value` is attention TFLOP/s over the whole step (FLOPs of the kept keys
only, 4*B*H*T_q*T_kv*D per launch; the time includes append/evict and similarity).  Besides the
headline fields the line carries
  modes            the same inputs under four policies -- vanilla (every layer keeps everything), the
                   benchmark's layer mix, every layer cache-efficient ({0,1} + window 2), every layer at the
                   paper's smallest budget ({0,1} + window 1) -- with ms per step, attention ms and KV bytes
                   each: the attention-latency comparison
  other_workloads  the other shapes the contract names (VAR-d16 stack at batch 32, VAR-d24 with ragged per-layer
                   policies at batch 64, Infinity-2B shape at batch 8, VAR-d30 at batch 128) and VAR-d30 at batch 512 (twice the largest batch the paper
                   reports; inputs and cache resident in one device's HBM), each with its own roofline object
(skipped with --quick, or when --workload / --mode select something else than the default).
"""
from __future__ import annotations

import argparse
import gc
import glob
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0          # MI355X HBM3E, published
PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
PROBE_SCALE = 5                # first step at which {0,1}+window 2 evicts a scale
COS_THRESHOLD = 0.5
EB = 2                         # bytes per element (bf16)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def measured_traffic(kernel, workload, mode, layout, borrow, fuse):
    """HBM bytes per launch of the dominant kernel from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary under
    profiles/ that was taken on exactly this kernel and configuration (a `bench-key:` line), else None."""
    want = {"kernel": kernel, "workload": workload, "mode": mode, "layout": layout, "borrow": str(int(borrow)), "fuse": str(int(fuse))}
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*hbm_traffic*.txt"))):
        for line in open(path):
            if not line.startswith("bench-key:"):
                continue
            kv = dict(x.split("=", 1) for x in line[len("bench-key:"):].split())
            if all(kv.get(k) == v for k, v in want.items()) and "traffic_bytes_per_launch" in kv:
                return int(kv["traffic_bytes_per_launch"])
    return None


class Inputs:
    """Synthetic Q, K, V of one workload, resident in HBM, plus output buffers and raw addresses."""

    def __init__(self, name, batch, dev):
        import torch
        import amskv_inputs as inp
        fn = {"var_d30": inp.config3, "var_d16": inp.config2, "var_d24": inp.config5, "infinity_2b": inp.config4}[name]
        w = fn(batch) if batch else fn()
        if name != "var_d30":
            w.name += "_b%d" % w.batch
        self.w, self.key = w, name
        B, H, D, L = w.batch, w.heads, w.head_dim, w.layers
        t0 = time.time()
        self.Q, self.K, self.V = [], [], []
        if name == "var_d30":
            rhos = inp.layer_rhos(L, inp.layer_seed(3, 999))
        for l in range(L):
            if name == "var_d30":
                q, k, v = inp.correlated_qkv(w.sides, B, H, D, "bf16", inp.layer_seed(w.config_id, l), rhos[l], device=dev)
            elif name == "var_d16":
                q, k, v = inp.correlated_qkv(w.sides, B, H, D, "bf16", inp.layer_seed(w.config_id, l), 0.8, device=dev)
            else:
                q, k, v = inp.iid_qkv(w.sides, B, H, D, "bf16", inp.layer_seed(w.config_id, l), device=dev)
            self.Q.append(q); self.K.append(k); self.V.append(v)
        self.O = [torch.empty(B, H, t, D, dtype=torch.bfloat16, device=dev) for t in w.tokens]
        torch.cuda.synchronize()
        log("%s: inputs %.1f GB in %.1f s" % (w.name, 3 * L * B * H * sum(w.tokens) * D * EB / 1e9, time.time() - t0))
        self.Kp = [[t.data_ptr() for t in self.K[l]] for l in range(L)]
        self.Vp = [[t.data_ptr() for t in self.V[l]] for l in range(L)]
        self.Qp = [[t.data_ptr() for t in self.Q[l]] for l in range(L)]
        self.Op = [t.data_ptr() for t in self.O]
        self.stream = int(torch.cuda.current_stream().cuda_stream)


def probe_policies(amskv, torch, x, dev):
    """The benchmark's layer mix: cache-demanding layers (mean cosine of Eq. 3 at the probe scale < 0.5) keep
    everything, the others the configuration's policy."""
    w = x.w
    B, H, D, L = w.batch, w.heads, w.head_dim, w.layers
    need = amskv.amskv_cache_required_bytes(1, H, D, w.sides, w.sides, B, 1, [(0, 0, True)])
    arena = torch.empty(need, dtype=torch.uint8, device=dev)
    prof = amskv.amskv_cache_create(1, H, D, w.sides, w.sides, B, 1, [(0, 0, True)], arena=arena)
    cos_layer = []
    for l in range(L):
        amskv.amskv_cache_reset(prof)
        for s in range(PROBE_SCALE + 1):
            amskv.amskv_append_scale(prof, 0, s, x.K[l][s], x.V[l][s])
        ck, _, _ = amskv.amskv_interscale_similarity(prof, 0, PROBE_SCALE, H, want_v=False, want_sums=False)
        cos_layer.append(sum(ck) / H)
    amskv.amskv_cache_destroy(prof)
    del arena
    pols = [(0, 0, True) if c < COS_THRESHOLD else w.policies[l] for l, c in enumerate(cos_layer)]
    log("mean cosine per layer:", " ".join("%.2f" % c for c in cos_layer))
    log("cache-demanding layers:", [l for l, p in enumerate(pols) if p[2]])
    return pols


def plan_trace(amskv, w, pols, budgets, layout, borrow, fuse, windows=None):
    """What every step attends to, moves and copies, from the library's own host logic on a plan-only cache
    (no device memory): per (layer, scale) the tokens attended, the tokens that changed their place in the arena
    and the tokens of the new scale written into it."""
    B, H, D, L, S = w.batch, w.heads, w.head_dim, w.layers, len(w.tokens)
    plan = amskv.amskv_cache_create(L, H, D, w.sides, w.sides, B, 1, pols, 0.0, layout, borrow_unretained=borrow,
                                    fuse_append=fuse, budgets=budgets, windows=windows)
    token_mode = budgets is not None or windows is not None
    kv_len = [[0] * S for _ in range(L)]
    moved = [[0] * S for _ in range(L)]
    copied = [[0] * S for _ in range(L)]
    try:
        for l in range(L):
            prev = {}
            for s in range(S):
                amskv.amskv_append_scale(plan, l, s)
                segs = amskv.amskv_cache_segments(plan, l)
                kv_len[l][s] = sum(x[3] for x in segs)            # the step's attention sees these (current scale included)
                if token_mode:
                    amskv.amskv_cache_settle(plan, l)             # the step's iteration of Algorithm 1
                    segs = amskv.amskv_cache_segments(plan, l)
                now = {(sc, first + i): off + i for sc, first, off, ln in segs if off >= 0 for i in range(ln)}
                for key, at in now.items():
                    if key not in prev:
                        copied[l][s] += 1
                    elif prev[key] != at:
                        moved[l][s] += 1
                prev = now
    finally:
        amskv.amskv_cache_destroy(plan)
    return kv_len, moved, copied


def step_accounting(w, t_kv, moved, copied, s, token_mode, fuse):
    """(attention FLOPs, algorithmic bytes of the attend call, algorithmic bytes of the append call) of one layer's step
    s, from the tokens the step attends to (`t_kv`, its own scale included) and the tokens its bookkeeping moves inside
    the arena or copies into it (plan_trace).  FLOPs: 4 T_q T_kv D per (b,h) -- the kept keys only.  Bytes of the
    attention: Q read, O written, K~ and V~ read once, plus what the same launch writes into the cache."""
    tokens, S = w.tokens, len(w.tokens)
    unit = w.head_dim * EB * w.batch * w.heads
    by = (2 * tokens[s] + 2 * t_kv) * unit
    roll = 2 * (2 * moved + 2 * copied) * unit                 # K and V: read + write what moves or is copied in
    if token_mode:
        aby = 0.0
        if s + 1 == S:
            pass                                   # the iteration after the last step never runs (reset)
        elif moved == 0 and copied == tokens[s]:
            by += 2 * copied * unit                # the scale fits untrimmed: the attend launch writes it as it streams it
        else:
            # the attend launch also writes the survivors to their new places (bf16, one workgroup per (b,h): every
            # step of these shapes), whichever way an Eq. 3 test decided on the device in front of it comes out
            by += 2 * (moved + copied) * unit
    elif fuse:
        by += 2 * copied * unit                    # the attend launch streams the scale anyway: only the write of K_s, V_s is extra
        aby = 2 * 2 * moved * unit
    else:
        aby = roll
    return 4.0 * w.batch * w.heads * tokens[s] * t_kv * w.head_dim, by, aby


def dominant_kernel_name(w, tokens):
    D = w.head_dim
    if D == 128:
        return "attend_bf16_kernel<128,1,4,32,3>"
    return "attend_bf16_kernel<64,1,8,64,4>" if max(tokens) > 128 else "attend_bf16_kernel<64,1,4,32,4>"


def measure(amskv, torch, x, dev, mode, pols, budgets, layout_name, borrow, fuse, steps, warmup, per_scale=False, n_inst=3,
            windows=None, graph_replay=True):
    """Timed steps, then instrumented passes with HIP events around every launch on the launch stream."""
    w = x.w
    B, H, D, L = w.batch, w.heads, w.head_dim, w.layers
    tokens, S = w.tokens, len(w.tokens)
    layout = amskv.AMSKV_LAYOUT_PLANNED if layout_name == "planned" else amskv.AMSKV_LAYOUT_COMPACT
    need = amskv.amskv_cache_required_bytes(L, H, D, w.sides, w.sides, B, 1, pols, 0.0, layout, borrow, fuse, budgets=budgets,
                                            windows=windows)
    arena = torch.empty(need, dtype=torch.uint8, device=dev)
    cache = amskv.amskv_cache_create(L, H, D, w.sides, w.sides, B, 1, pols, 0.0, layout, arena=arena,
                                     borrow_unretained=borrow, fuse_append=fuse, budgets=budgets, windows=windows)
    token_mode = budgets is not None or windows is not None
    probe = PROBE_SCALE if S > PROBE_SCALE else S - 1
    Kp, Vp, Qp, Op, stream = x.Kp, x.Vp, x.Qp, x.Op, x.stream

    def one_step(timers=None):
        amskv.amskv_cache_reset(cache)
        for s in range(S):
            for l in range(L):
                if timers is None:
                    amskv.amskv_append_scale(cache, l, s, Kp[l][s], Vp[l][s], stream)
                    amskv.amskv_attend(cache, l, s, Qp[l][s], Op[s], stream)
                else:
                    e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
                    e[0].record()
                    amskv.amskv_append_scale(cache, l, s, Kp[l][s], Vp[l][s], stream)
                    e[1].record()
                    amskv.amskv_attend(cache, l, s, Qp[l][s], Op[s], stream)
                    e[2].record()
                    timers.append((l, s, e))
            if s == probe and probe >= 1 and not token_mode:
                for l in range(L):
                    amskv.amskv_interscale_similarity_enqueue(cache, l, s, want_v=False, stream=stream)
        if probe >= 1 and not token_mode:   # the scores of all layers: one transfer, one wait per step
            amskv.amskv_interscale_similarity_collect(cache, L, H, want_v=False, want_sums=False, stream=stream)

    for _ in range(warmup):
        one_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        one_step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps

    # The same device work recorded once into a HIP graph and replayed (scale-window mode enqueues kernels only; the
    # host side of the calls -- kept sets, slots, arguments -- then runs once, at capture).  Reported beside the
    # headline, never as it: what a serving loop with fixed buffers would see.
    graph_ms = None
    if not token_mode and graph_replay:
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            st = int(torch.cuda.current_stream().cuda_stream)
            amskv.amskv_cache_reset(cache)
            for s in range(S):
                for l in range(L):
                    amskv.amskv_append_scale(cache, l, s, Kp[l][s], Vp[l][s], st)
                    amskv.amskv_attend(cache, l, s, Qp[l][s], Op[s], st)
                if s == probe and probe >= 1:
                    for l in range(L):
                        amskv.amskv_interscale_similarity_enqueue(cache, l, s, want_v=False, stream=st)
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / steps
        del graph

    expanded = []
    forced = budgets
    if budgets is not None:
        # which layers the Eq. 3 test expanded is read back from the cache; the plan-only trace repeats those decisions
        expanded = [amskv.amskv_cache_budget_tokens(cache, l) == budgets[l][1] for l in range(L)]
        forced = [(a, b, c, 2.0 if expanded[l] else -2.0) for l, (a, b, c, _) in enumerate(budgets)]
        log("layers whose budget the Eq. 3 test expanded:", [l for l in range(L) if expanded[l]])
    kv_len, moved, copied = plan_trace(amskv, w, pols, forced, layout, borrow, fuse, windows)
    flops = sum(step_accounting(w, kv_len[l][s], moved[l][s], copied[l][s], s, token_mode, fuse)[0] for l in range(L) for s in range(S))
    held = sum(amskv.amskv_cache_bytes_held(cache, l, True) for l in range(L))
    held_paper = sum(amskv.amskv_cache_bytes_held(cache, l, False) for l in range(L))

    # the instrumented passes create two event objects per call: keep the interpreter's collector out of the intervals
    # (a generation-2 pass between two event records once showed up as a 30 ms "append" that launches nothing)
    timers = []
    gc.collect()
    gc.disable()
    try:
        for _ in range(n_inst):
            one_step(timers)
            torch.cuda.synchronize()
    finally:
        gc.enable()
    dom_rows = 128 if D == 64 and max(tokens) > 128 else 32    # launches of the dominant kernel: T_q above this
    dom_t = dom_bytes = dom_flops = 0.0
    dom_n = 0
    att_t = app_t = att_bytes = app_bytes = 0.0
    scale_rows = [[0.0, 0.0, 0.0, 0.0] for _ in range(S)]
    for l, s, e in timers:
        ta, tt = e[0].elapsed_time(e[1]) * 1e-3, e[1].elapsed_time(e[2]) * 1e-3
        fl, by, aby = step_accounting(w, kv_len[l][s], moved[l][s], copied[l][s], s, token_mode, fuse)
        att_t += tt; app_t += ta; att_bytes += by; app_bytes += aby
        r = scale_rows[s]
        r[0] += ta; r[1] += tt; r[2] += fl; r[3] += by
        if tokens[s] > dom_rows:
            dom_t += tt; dom_bytes += by; dom_flops += fl; dom_n += 1
    if dom_n == 0:
        dom_t, dom_bytes, dom_flops, dom_n = att_t, att_bytes, flops * n_inst, len(timers)
    dom_t, dom_bytes, dom_flops, dom_n = dom_t / n_inst, dom_bytes / n_inst, dom_flops / n_inst, dom_n // n_inst
    att_t, app_t, att_bytes, app_bytes = att_t / n_inst, app_t / n_inst, att_bytes / n_inst, app_bytes / n_inst
    scale_rows = [[v / n_inst for v in row] for row in scale_rows]
    if per_scale:
        log("scale  T_q  append_ms attend_ms  TFLOP/s   GB/s(attend)")
        for s in range(S):
            a, t, fl, by = scale_rows[s]
            log("%5d %4d %9.3f %9.3f %8.1f %8.1f" % (s, tokens[s], a * 1e3, t * 1e3, fl / t / 1e12, by / t / 1e9))
        log("attend total %.2f ms, append total %.2f ms" % (att_t * 1e3, app_t * 1e3))

    dom_name = dominant_kernel_name(w, tokens)
    if budgets is not None:   # the timed interval of an attend call holds the step's Eq. 3 test too
        dom_name += " + Eq. 3 test kernels of the step"
    ai = dom_flops / dom_bytes
    if ai < PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9):
        roof = {"bound": "hbm", "achieved": dom_bytes / dom_t / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s"}
    else:
        roof = {"bound": "mfma", "achieved": dom_flops / dom_t / 1e12, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = measured_traffic(dom_name, w.name, mode, layout_name, borrow, fuse)
    roof.update({"kernel": dom_name, "launches": dom_n, "avg_launch_ms": dom_t / dom_n * 1e3,
                 "algorithmic_bytes_per_launch": dom_bytes / dom_n, "flops_per_launch": dom_flops / dom_n,
                 "arithmetic_intensity": ai, "tflops": dom_flops / dom_t / 1e12,
                 "frac_of_bf16_mfma_peak": dom_flops / dom_t / 1e12 / PEAK_BF16_TFLOPS,
                 "frac_of_min_roof": (dom_flops / dom_t) / min(PEAK_BF16_TFLOPS * 1e12, ai * PEAK_HBM_GBS * 1e9)})
    res = {"ms_per_step": ms_per_step, "flops": flops, "tflops": flops / (ms_per_step * 1e-3) / 1e12,
           "attend_ms": att_t * 1e3, "append_ms": app_t * 1e3, "append_gbs": app_bytes / max(app_t, 1e-9) / 1e9,
           "held": held, "held_paper": held_paper, "vanilla_held": 2 * EB * B * H * D * sum(tokens) * L, "arena": need,
           "roofline": roof, "expanded": expanded, "kv_len": kv_len, "cache": cache, "arena_tensor": arena,
           "graph_ms": graph_ms,
           "pols": pols, "probe": probe}
    return res


def release(amskv, res):
    amskv.amskv_cache_destroy(res.pop("cache"))
    res.pop("arena_tensor")


def standalone_append(amskv, torch, x, dev, pols):
    """The evict + compact + append kernels by themselves: one instrumented pass over a cache in the copying
    configuration (COMPACT layout, nothing borrowed or fused), for their HBM rate."""
    w = x.w
    B, H, D, L = w.batch, w.heads, w.head_dim, w.layers
    tokens, S = w.tokens, len(w.tokens)
    need = amskv.amskv_cache_required_bytes(L, H, D, w.sides, w.sides, B, 1, pols)
    arena = torch.empty(need, dtype=torch.uint8, device=dev)
    cache = amskv.amskv_cache_create(L, H, D, w.sides, w.sides, B, 1, pols, arena=arena)
    _, moved, copied = plan_trace(amskv, w, pols, None, amskv.AMSKV_LAYOUT_COMPACT, False, False)
    ev = []
    for s in range(S):
        for l in range(L):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            amskv.amskv_append_scale(cache, l, s, x.Kp[l][s], x.Vp[l][s], x.stream)
            e1.record()
            ev.append((l, s, e0, e1))
    torch.cuda.synchronize()
    t = b = 0.0
    for l, s, e0, e1 in ev:
        if tokens[s] >= 64:            # launches large enough to be bandwidth- rather than latency-bound
            t += e0.elapsed_time(e1) * 1e-3
            b += 2 * (2 * moved[l][s] + 2 * copied[l][s]) * D * EB * B * H
    amskv.amskv_cache_destroy(cache)
    del arena
    return {"what": "evict + compact + append kernels, COMPACT layout, nothing borrowed or fused, scales with T_s >= 64, "
                    "read+write bytes", "gbs": b / max(t, 1e-9) / 1e9, "frac_of_hbm_peak": b / max(t, 1e-9) / 1e9 / PEAK_HBM_GBS,
            "ms": t * 1e3}


def density_probe(amskv, torch, x, res):
    """The attention-density by-product (Section 4.1) of the last step: one enqueued call per layer, the masses of all
    layers read back with one wait at the end."""
    w = x.w
    B, H, D, L = w.batch, w.heads, w.head_dim, w.layers
    S = len(w.tokens)
    cache = res["cache"]
    outs = torch.empty(L, H * amskv.AMSKV_MAX_SCALES, dtype=torch.float32, device="cuda")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    amskv.amskv_attention_density_enqueue(cache, 0, S - 1, x.Qp[0][S - 1], outs[0], x.stream)   # warm-up
    e0.record()
    lens = [amskv.amskv_attention_density_enqueue(cache, l, S - 1, x.Qp[l][S - 1], outs[l], x.stream) for l in range(L)]
    e1.record()
    torch.cuda.synchronize()
    d_ms = e0.elapsed_time(e1) / L
    d_fl = sum(2.0 * B * H * w.tokens[S - 1] * res["kv_len"][l][S - 1] * D for l in range(L)) / L
    last = outs[L - 1].cpu().numpy().reshape(H, amskv.AMSKV_MAX_SCALES)[0, : len(lens[-1])]
    # the same masses as a by-product of the step's own attention launch (amskv_attend_density) against that launch alone
    outs2 = torch.empty_like(outs)
    t = []
    for with_density in (False, True, False, True):
        e0.record()
        for l in range(L):
            if with_density:
                amskv.amskv_attend_density(cache, l, S - 1, x.Qp[l][S - 1], x.Op[S - 1], outs2[l], x.stream)
            else:
                amskv.amskv_attend(cache, l, S - 1, x.Qp[l][S - 1], x.Op[S - 1], x.stream)
        e1.record()
        torch.cuda.synchronize()
        t.append(e0.elapsed_time(e1) / L)
    n_max = max(len(n) for n in lens)
    a = outs.view(L, H, amskv.AMSKV_MAX_SCALES)[:, :, :n_max].double()
    b = outs2.view(L, H, amskv.AMSKV_MAX_SCALES)[:, :, :n_max].double()
    ok = torch.tensor([[i < len(n) for i in range(n_max)] for n in lens], device=a.device)[:, None, :]
    dev_rel = float((((a - b).abs() / a.abs().clamp_min(1e-30)) * ok).max())
    return {"what": "per-head softmax mass per cached token of each kept scale, last step, one enqueued call per layer "
                    "(two kernels, the masses written straight into the caller's buffer; one wait for all layers)", "ms_per_call": d_ms,
            "tflops_qk": d_fl / (d_ms * 1e-3) / 1e12,
            "last_layer_head0_density_per_kept_scale": [round(float(m) / n, 4) for m, n in zip(last, lens[-1])],
            "as_by_product_of_the_attention_launch": {
                "what": "amskv_attend_density against amskv_attend at the last step, ms per layer call (second of two passes each)",
                "attend_ms": t[2], "attend_density_ms": t[3], "extra_ms": t[3] - t[2],
                "max_rel_difference_to_the_stand_alone_masses": dev_rel}}


def workload_record(w, mode, layout_name, borrow, fuse, res):
    return {"workload": w.name, "mode": mode, "layout": layout_name, "borrow_unretained": int(borrow), "fuse_append": int(fuse),
            "layers": w.layers, "heads": w.heads, "head_dim": w.head_dim, "batch": w.batch, "tokens": sum(w.tokens),
            "ms_per_step": res["ms_per_step"], "ms_per_image": res["ms_per_step"] / w.batch, "tflops": res["tflops"],
            "frac_of_bf16_mfma_peak": res["tflops"] / PEAK_BF16_TFLOPS, "attend_ms_per_step": res["attend_ms"],
            "kv_bytes_held": res["held"], "kv_bytes_held_excluding_current_scale": res["held_paper"],
            "kv_bytes_vanilla": res["vanilla_held"], "roofline": res["roofline"],
            "ms_per_step_as_replayed_hip_graph": res["graph_ms"]}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="var_d30", choices=["var_d30", "var_d16", "var_d24", "infinity_2b"])
    ap.add_argument("--batch", type=int, default=0, help="0 = the configuration's batch")
    ap.add_argument("--mode", default="amskv", choices=["amskv", "vanilla", "efficient", "token_budget", "swa", "sta"],
                    help="amskv: per-layer scale windows picked from the similarity probe (the default, the contract's "
                         "workload); vanilla: every layer keeps everything; efficient: every layer gets the configuration's "
                         "cache-efficient policy; token_budget: Algorithms 1 and 2 literally, budgets in tokens, the Eq. 3 "
                         "test and the budget expansion run inside the step; swa / sta: the sliding-window and sink + window "
                         "kept sets of the paper's comparison at 75 %% compression (a quarter of the schedule's tokens, "
                         "sta with the first two scales as sinks), token-granular, structure only")
    ap.add_argument("--layout", default="planned", choices=["compact", "planned"],
                    help="planned (default): every scale has a fixed slot, eviction moves nothing; compact: kept "
                         "scales stay back to back, eviction slides the survivors down")
    ap.add_argument("--no-borrow", action="store_true",
                    help="copy every appended scale into the arena, also the ones no later step reads "
                         "(default: borrow_unretained=1, the final scale is attended in place as in Algorithm 1)")
    ap.add_argument("--no-fuse", action="store_true",
                    help="copy retained scales in amskv_append_scale (default: fuse_append=1, the attend call of the "
                         "step fills the scale's slot while it streams the scale)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--quick", action="store_true", help="headline measurement only: no modes, no other workloads")
    ap.add_argument("--path-only", action="store_true",
                    help="with --quick: nothing but the passes of the path itself (no stand-alone append pass, no density "
                         "probe, no graph replay), so that a profiler's per-kernel means are means over the path's own launches")
    ap.add_argument("--per-scale", action="store_true", help="print a per-scale timing table to stderr")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 4 GiB device copy five times (reference dispatch of known size for "
                         "scaling the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus %d is not supported (every (layer, batch, head) "
              "unit is independent, so more GPUs would shard the batch with no exchange)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2511_16047_amd as amskv

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    amskv.load_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.copy_calibration:
        a = torch.ones(1 << 30, dtype=torch.int32, device=dev)
        b = torch.empty_like(a)
        for _ in range(5):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": 4 << 30, "copy_bytes_written": 4 << 30, "repeats": 5}))
        return

    layout_name = args.layout
    borrow, fuse = not args.no_borrow, not args.no_fuse
    x = Inputs(args.workload, args.batch, dev)
    w = x.w
    tokens, S, L, H, D, B = w.tokens, len(w.tokens), w.layers, w.heads, w.head_dim, w.batch
    budgets = windows = None
    mix = probe_policies(amskv, torch, x, dev) if args.workload == "var_d30" and args.mode in ("amskv",) else None
    if args.mode == "token_budget":
        # Section 5 set-up read as token counts: condensed = the first two scales, C_min = condensed + the
        # penultimate scale, C_max = condensed + the two scales before the last; the cached tokens stay one
        # contiguous run (COMPACT), the current scale is always read in place
        c_cds = tokens[0] + tokens[1]
        budgets = [(c_cds + tokens[-2], c_cds + tokens[-3] + tokens[-2], c_cds, COS_THRESHOLD)] * L
        layout_name, borrow, fuse = "compact", False, False
        pols = None
    elif args.mode in ("swa", "sta"):
        windows = [(sum(tokens) // 4, tokens[0] + tokens[1] if args.mode == "sta" else 0)] * L
        layout_name, borrow, fuse = "compact", False, False
        pols = None
    elif args.mode == "vanilla":
        pols = [(0, 0, True)] * L
    elif args.mode == "efficient" or mix is None:
        pols = list(w.policies)
    else:
        pols = mix

    res = measure(amskv, torch, x, dev, args.mode, pols, budgets, layout_name, borrow, fuse, args.steps, args.warmup,
                  per_scale=args.per_scale, windows=windows, graph_replay=not args.path_only)
    sa = None if args.path_only else standalone_append(amskv, torch, x, dev, pols if pols is not None else list(w.policies))
    dens = density_probe(amskv, torch, x, res) if pols is not None and not args.path_only else None
    roof = res["roofline"]

    out = {
        "metric": "AMS-KV attention TFLOP/s + ms per image at VAR-d30 b=256; KV bytes held",
        "value": res["tflops"], "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "mode": args.mode, "layout": layout_name, "borrow_unretained": int(borrow),
                   "fuse_append": int(fuse), "layers": L, "heads": H, "head_dim": D, "batch": B, "tokens": sum(tokens), "scales": S,
                   "cache_demanding_layers": sum(res["expanded"]) if budgets is not None else sum(1 for p in (pols or []) if p[2]),
                   "probe_scale": res["probe"],
                   **({"budgets_c_min_c_max_c_cds_theta": list(budgets[0])} if budgets is not None else {}),
                   **({"window_tokens_and_sinks": list(windows[0])} if windows is not None else {})},
        "ms_per_image": res["ms_per_step"] / B,
        "ms_per_step_as_replayed_hip_graph": res["graph_ms"],
        "kv_bytes_held": res["held"], "kv_bytes_held_excluding_current_scale": res["held_paper"],
        "kv_bytes_vanilla": res["vanilla_held"], "kv_reduction": 1.0 - res["held"] / res["vanilla_held"],
        "arena_bytes": res["arena"], "attention_flops_per_step": res["flops"],
        "attend_ms_per_step": res["attend_ms"], "append_ms_per_step": res["append_ms"], "append_gbs": res["append_gbs"],
        "standalone_append": sa,
        "attention_density": dens,
        "roofline": roof,
        "binding_roof": "HBM: at head dim 64 and T_q <= 256 the arithmetic intensity (T_q*T_kv/(T_q+T_kv) flop/byte) is below the "
                        "chip's ridge, so the HBM roof caps the dominant kernel at frac_of_min_roof = 1 long before bf16 MFMA peak; "
                        "roofline.frac is the fraction of that HBM roof" if roof["bound"] == "hbm" else "MFMA",
        "paper_context": {"kv_reduction_up_to": 0.8483, "self_attention_latency_reduction": 0.6048,
                          "var_d30_b256": "44.94 GB KV, 23.88 img/s whole model", "hardware": "NVIDIA A100-80GB, FlashAttention-2"},
    }
    kv_len0 = res["kv_len"][0]
    budget0 = None if budgets is None else (budgets[0], res["expanded"][0])
    release(amskv, res)

    full = not args.quick and args.workload == "var_d30" and args.mode == "amskv" and not args.batch
    if full:
        # ---------------- the same inputs under the other two policies: the attention-latency comparison
        modes = {"amskv": {"what": "the benchmark's layer mix (cache-demanding layers keep everything)",
                           "ms_per_step": out["ms_per_step"], "attend_ms_per_step": out["attend_ms_per_step"],
                           "kv_bytes_held": out["kv_bytes_held"], "kv_bytes_held_excluding_current_scale": res["held_paper"],
                           "attention_flops_per_step": res["flops"], "cache_demanding_layers": out["config"]["cache_demanding_layers"]}}
        for name, p, what in (("vanilla", [(0, 0, True)] * L, "every layer keeps every scale"),
                              ("efficient", list(w.policies), "every layer condensed {0,1} + window 2"),
                              ("efficient_window_1", [(2, 1, False)] * L,
                               "every layer condensed {0,1} + the one preceding scale: the paper's C_min (first two scales + "
                               "penultimate scale) expressed in scales")):
            r = measure(amskv, torch, x, dev, name, p, None, layout_name, borrow, fuse, max(3, args.steps // 3), 1, n_inst=2)
            release(amskv, r)
            modes[name] = {"what": what, "ms_per_step": r["ms_per_step"], "attend_ms_per_step": r["attend_ms"],
                           "kv_bytes_held": r["held"], "kv_bytes_held_excluding_current_scale": r["held_paper"],
                           "attention_flops_per_step": r["flops"], "cache_demanding_layers": sum(1 for q in p if q[2])}
        van = modes["vanilla"]
        for name in ("amskv", "efficient", "efficient_window_1"):
            m = modes[name]
            m["attention_latency_reduction_vs_vanilla"] = 1.0 - m["attend_ms_per_step"] / van["attend_ms_per_step"]
            m["kv_reduction_vs_vanilla"] = 1.0 - m["kv_bytes_held"] / van["kv_bytes_held"]
            m["kv_reduction_vs_vanilla_excluding_current_scale"] = 1.0 - m["kv_bytes_held_excluding_current_scale"] / van["kv_bytes_held_excluding_current_scale"]
        out["modes"] = modes

    # ---------------- the oracle, timed on the host cores, on a bounded sample of the same workload
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, pols, x.K, x.V, x.Q, tokens, H, D, kv_len0, out["attention_flops_per_step"], budget0,
                                           None if windows is None else windows[0])

    if full:
        # ---------------- the other shapes the contract names, each with its own roofline object
        del x
        torch.cuda.empty_cache()
        others = []
        for key, batch, st in (("var_d30", 128, 5), ("var_d30", 512, 3), ("var_d16", 0, 10), ("var_d24", 0, 5), ("infinity_2b", 0, 3)):
            y = Inputs(key, batch, dev)
            p = probe_policies(amskv, torch, y, dev) if key == "var_d30" else list(y.w.policies)
            r = measure(amskv, torch, y, dev, "amskv", p, None, layout_name, borrow, fuse, st, 1, n_inst=2)
            release(amskv, r)
            others.append(workload_record(y.w, "amskv", layout_name, borrow, fuse, r))
            if key == "var_d24":
                # the sweep the configuration is named for: every layer at (condensed c, window w), all twelve corners
                sweep = []
                for cds in (1, 2, 3):
                    for win in (1, 2, 3, 4):
                        q = measure(amskv, torch, y, dev, "amskv", [(cds, win, False)] * y.w.layers, None, layout_name, borrow, fuse,
                                    3, 1, n_inst=1, graph_replay=False)
                        release(amskv, q)
                        sweep.append({"condensed": cds, "window": win, "ms_per_step": q["ms_per_step"], "tflops": q["tflops"],
                                      "kv_bytes_held": q["held"], "frac_of_hbm_roof": q["roofline"]["frac"]})
                others[-1]["policy_sweep"] = sweep
            del y, r
            torch.cuda.empty_cache()
        out["other_workloads"] = others
    print(json.dumps(out), flush=True)


def cpu_baseline(w, pols, K, V, Q, tokens, H, D, kv_len0, step_flops, budget0=None, window0=None):
    """The oracle as it stands, on (layer 0, the first few batch rows, all heads, all scales)."""
    import numpy as np
    from oracle import amskv_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    S = len(tokens)
    l = 0
    done_flops, elapsed, nb = 0.0, 0.0, 0
    budget = 12.0
    b = 0
    while elapsed < budget and b < w.batch:
        nb_now = 1 if b == 0 else min(max(1, int(nb * (budget - elapsed) / max(elapsed, 1e-3))), 8, w.batch - b)
        q = [t[b:b + nb_now].double().cpu().numpy() for t in Q[l]]
        k = [t[b:b + nb_now].double().cpu().numpy() for t in K[l]]
        v = [t[b:b + nb_now].double().cpu().numpy() for t in V[l]]
        t0 = time.perf_counter()
        if window0 is not None:
            cat = lambda xs: np.concatenate(xs, axis=-2)
            orc.masked_attention(cat(q), cat(k), cat(v), orc.token_window_allow_mask(tokens, window0[0], window0[1]))
        elif budget0 is not None:
            (c_min, c_max, c_cds, _), grew = budget0
            trace = orc.alg1_cache_trace(tokens, c_min, c_max, c_cds, [grew] * S)
            cat = lambda xs: np.concatenate(xs, axis=-2)
            orc.masked_attention(cat(q), cat(k), cat(v), orc.alg1_allow_mask(tokens, trace))
        else:
            orc.attend_all_steps(q, k, v, tokens, pols[l])
            for s in range(S):
                orc.cache_contents(k, pols[l], s)
                orc.cache_contents(v, pols[l], s)
        if S > PROBE_SCALE:
            sd = (w.sides[PROBE_SCALE],) * 2, (w.sides[PROBE_SCALE - 1],) * 2
            orc.interscale_similarity(k[PROBE_SCALE], k[PROBE_SCALE - 1], sd[0], sd[1])
        elapsed += time.perf_counter() - t0
        done_flops += sum(4.0 * nb_now * H * tokens[s] * kv_len0[s] * D for s in range(S))
        b += nb_now
        nb += nb_now
    rate = done_flops / elapsed
    return {"value": rate / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": "layer 0, batch rows 0..%d, all %d heads, all %d scales (attention over the explicit mask, "
                      "cache contents, probe-scale similarity); %.1f s measured" % (nb - 1, H, S, elapsed),
            "extrapolated_seconds_per_step": step_flops / rate,
            "extrapolation": "the units (layer, batch row, head) are independent and equally sized per layer policy, so the "
                             "whole step (%d layers x batch %d) is the measured rate applied to its %.3e attention FLOPs"
                             % (w.layers, w.batch, step_flops)}


if __name__ == "__main__":
    main()
