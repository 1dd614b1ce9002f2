#!/usr/bin/env python3
"""Benchmark of the MaskKV eviction hot path on one MI355X.

One step = one layer of the headline long-context configuration (32 heads x head_dim 128, bf16,
P = 32768 prompt tokens, 256 mask queries, 256 kept KV pairs per head on average with a 2:1
per-head split, pool window 7) pushed through the whole path:
    maskkv_score -> maskkv_select -> maskkv_compact -> maskkv_attend.
Steps rotate over several resident layers with independent seeds so that nothing is served from
cache by accident.  Inputs are synthetic (Gaussian with planted prompt positions), generated on
the device before the timed region.  Shapes, planting and budgets come from synth.CONFIGS.

Prints ONE JSON line.  `value` is the metric's own definition: prompt tokens scored + evicted per
second per layer = P / (t_score + t_select + t_compact), the three calls bracketed by HIP events
inside the timed region; `ms_per_step` is the wall time of the whole step (attention included).
The line also carries per-call timings (mean, median, minimum over the timed steps), compressed- and
full-cache attention TFLOP/s, a roofline object for the dominant kernel (score pass 1, bracketed by
HIP events on the launch stream inside the timed region) with the whole scoring call beside it, the
same calls on peaky logits, the other configurations (a single 4k-prompt layer, the 8k-prompt
32-layer stack with its budget schedule, the 32k-prompt stack with on-device head budgets, the
batched ragged configuration), probes of what the box sustains, and the CPU oracle timed on bounded
samples.
"""
from __future__ import annotations

import argparse
import ctypes as ct
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16
HBM_PEAK_GBS = 8000.0
# HBM bytes read + written by one launch of score pass 1 at the 32k prompt: rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE,
# each scaled by what it reads for a copy of known size (profiles/score_pass1_c4_hbm_traffic.md).  Other workloads: null.
SCORE_PASS1_TRAFFIC_BYTES = {"C4": 141373.0 * 1024 * 2.0 + 1126.0 * 1024}


def workload(name: str) -> dict:
    """Shape, planting and budgets of a named benchmark configuration (one definition: synth.CONFIGS)."""
    from paper_2510_09309_amd import synth
    cfg = dict(synth.CONFIGS[name])
    cfg["name"] = name
    return cfg


class HipEvents:
    """Raw HIP events (created through the HIP runtime already loaded by torch) for stage timing."""

    def __init__(self):
        path = None
        with open("/proc/self/maps") as f:  # the HIP runtime instance torch and libmaskkv.so already share
            for line in f:
                if "libamdhip64" in line:
                    path = line.split()[-1]
                    break
        assert path, "HIP runtime is not loaded"
        self.hip = ct.CDLL(path)
        self.hip.hipEventElapsedTime.argtypes = [ct.POINTER(ct.c_float), ct.c_void_p, ct.c_void_p]
        self.hip.hipEventCreate.argtypes = [ct.POINTER(ct.c_void_p)]
        self.hip.hipEventDestroy.argtypes = [ct.c_void_p]
        self.hip.hipEventRecord.argtypes = [ct.c_void_p, ct.c_void_p]

    def create(self) -> int:
        ev = ct.c_void_p()
        rc = self.hip.hipEventCreate(ct.byref(ev))
        assert rc == 0, f"hipEventCreate failed: {rc}"
        return ev.value

    def record(self, ev: int, stream) -> None:
        rc = self.hip.hipEventRecord(ct.c_void_p(ev), ct.c_void_p(stream.cuda_stream))
        assert rc == 0, f"hipEventRecord failed: {rc}"

    def elapsed_ms(self, a: int, b: int) -> float:
        ms = ct.c_float()
        rc = self.hip.hipEventElapsedTime(ct.byref(ms), ct.c_void_p(a), ct.c_void_p(b))
        assert rc == 0, f"hipEventElapsedTime failed: {rc}"
        return float(ms.value)

    def destroy(self, ev: int) -> None:
        self.hip.hipEventDestroy(ct.c_void_p(ev))


def stats(ms) -> dict:
    a = np.asarray(ms, dtype=np.float64)
    return {"mean": float(a.mean()), "median": float(np.median(a)), "min": float(a.min())}


def device_layer(torch, cfg, layer, sigma=1.0):
    """Q [1,H,n_m,d], K, V [1,H,N,d] bf16 on the device: Gaussian * sigma / sqrt(d), unit direction u_h added to all
    mask queries, amplitude*u_h added to n_planted random prompt keys per head (same recipe as synth.make_layer)."""
    g = torch.Generator(device="cuda")
    g.manual_seed(cfg["seed"] + layer)
    H, d, P, n_m = cfg["H"], cfg["d"], cfg["P"], cfg["n_m"]
    N = P + n_m
    s = sigma / d ** 0.5
    Q = torch.randn((1, H, n_m, d), generator=g, device="cuda", dtype=torch.float32) * s
    K = torch.randn((1, H, N, d), generator=g, device="cuda", dtype=torch.float32) * s
    V = torch.randn((1, H, N, d), generator=g, device="cuda", dtype=torch.float32) * s
    u = torch.randn((H, d), generator=g, device="cuda", dtype=torch.float32)
    u = u / u.norm(dim=1, keepdim=True)
    Q += u[None, :, None, :]
    for h in range(H):
        pos = torch.randperm(P, generator=g, device="cuda")[:cfg["n_planted"]]
        K[0, h, pos] += cfg["amplitude"] * u[h]
    return Q.to(torch.bfloat16), K.to(torch.bfloat16), V.to(torch.bfloat16)


class Path:
    """Buffers and workspaces of one single-sequence configuration, and the calls of the path on resident layer i."""

    def __init__(self, torch, mk, cfg, layers, capacity):
        self.mk, self.cfg, self.layers = mk, cfg, layers
        self.row_lse = None            # per resident layer: natural-log row normalisers, if scoring is to use them
        H, d, P, n_m = cfg["H"], cfg["d"], cfg["P"], cfg["n_m"]
        self.desc = mk.Desc(B=1, H=H, d=d, dtype=mk.MASKKV_BF16, n_resp=n_m, P_max=P)
        self.resp = [(mk.tensor_view(K, seq_start=[P]), mk.tensor_view(V, seq_start=[P])) for (_, K, V) in layers]
        self.stride = (P + 63) // 64 * 64
        dev = dict(device="cuda")
        self.cap = capacity
        self.scores = torch.empty((H, self.stride), dtype=torch.float32, **dev)
        self.mass = torch.empty(H, dtype=torch.float32, **dev)
        self.idx = torch.empty(capacity, dtype=torch.int32, **dev)
        self.cu = torch.empty(H + 1, dtype=torch.int32, **dev)
        self.Kc = torch.empty((capacity, d), dtype=torch.bfloat16, **dev)
        self.Vc = torch.empty_like(self.Kc)
        self.O = torch.empty((1, H, n_m, d), dtype=torch.bfloat16, **dev)
        self.Of = torch.empty_like(self.O)
        ws = lambda n: torch.empty(max(n, 256), dtype=torch.uint8, **dev)
        self.ws_score = ws(mk.maskkv_score_workspace_bytes(self.desc))
        self.ws_sel = ws(mk.maskkv_select_workspace_bytes(self.desc))
        self.ws_att = ws(mk.maskkv_attend_workspace_bytes(self.desc, False))
        self.ws_full = ws(mk.maskkv_attend_workspace_bytes(self.desc, True))

    def score(self, i, stream, marks=None, bb=None):
        Q, K, _ = self.layers[i % len(self.layers)]
        if self.row_lse is not None:   # the second scoring pass alone, from given row normalisers
            self.mk.maskkv_score_given_lse(self.desc, Q, K, 0.0, self.row_lse[i % len(self.layers)], self.scores,
                                           self.stride, self.mass, self.ws_score, stream)
        elif marks is None:
            self.mk.maskkv_score(self.desc, Q, K, 0.0, self.scores, self.stride, self.mass, self.ws_score, stream)
        else:   # the same launches, with events recorded around the passes
            bb.maskkv_bench_score_marked(self.desc, Q, K, 0.0, self.scores, self.stride, self.mass, self.ws_score,
                                         marks, stream)

    def select(self, i, budgets, stream):
        self.mk.maskkv_select(self.desc, self.scores, self.stride, self.cfg["window"], self.mk.POOL_MEAN, budgets,
                              self.idx, self.cu, self.cap, self.ws_sel, stream)

    def compact(self, i, stream):
        _, K, V = self.layers[i % len(self.layers)]
        self.mk.maskkv_compact(self.desc, K, V, self.idx, self.cu, self.cap, self.Kc, self.Vc, stream)

    def attend(self, i, stream):
        Q = self.layers[i % len(self.layers)][0]
        Kr, Vr = self.resp[i % len(self.layers)]
        self.mk.maskkv_attend(self.desc, Q, self.Kc, self.Vc, self.cu, self.cap, Kr, Vr, 0.0, self.O, None,
                              self.ws_att, stream)

    def attend_full(self, i, stream):
        Q, K, V = self.layers[i % len(self.layers)]
        self.mk.maskkv_attend_full(self.desc, Q, K, V, 0.0, self.Of, None, self.ws_full, stream)


def timed_steps(torch, hev, path, budgets, steps, warmup, bb, every_call=False):
    """`warmup` untimed steps, then exactly `steps` whole-path steps timed by the wall clock, with HIP events on the
    launch stream inside the region.  An event between two kernels costs a few microseconds (the second kernel
    starts only after the event has been processed; kernels enqueued back to back start within 10 ns of each other),
    so the region proper records three per step: at the start of the step, after score pass 1, and after compact.
    `every_call` also brackets score, select, compact and attend separately (used for the per-call breakdown, not for
    the headline)."""
    stream = torch.cuda.current_stream()
    for i in range(warmup):
        path.score(i, stream)
        path.select(i, budgets, stream)
        path.compact(i, stream)
        path.attend(i, stream)
    two_pass = path.row_lse is None   # (the mark after pass 1 exists only in the two-pass scoring call)
    # per step: 0 start, 2 after pass 1, 3 scored, 4 selected, 5 gathered; one more event closes the last step
    ev = [[hev.create() for _ in range(6)] for _ in range(steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        e = ev[i]
        hev.record(e[0], stream)
        path.score(i, stream, marks=(0, e[2], 0, 0) if two_pass else None, bb=bb)
        if every_call:
            hev.record(e[3], stream)
        path.select(i, budgets, stream)
        if every_call:
            hev.record(e[4], stream)
        path.compact(i, stream)
        hev.record(e[5], stream)
        path.attend(i, stream)
    hev.record(ev[steps][0], stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    span = lambda a, b: [hev.elapsed_ms(e[a], e[b]) for e in ev[:steps]]
    out = {"wall_ms_per_step": wall_ms, "evict": span(0, 5),
           "attend": [hev.elapsed_ms(ev[i][5], ev[i + 1][0]) for i in range(steps)],
           "step": [hev.elapsed_ms(ev[i][0], ev[i + 1][0]) for i in range(steps)]}
    if two_pass:
        out["pass1"] = span(0, 2)
    if every_call:
        out.update({"score": span(0, 3), "select": span(3, 4), "compact": span(4, 5)})
    for e in ev:
        for x in e:
            hev.destroy(x)
    return out


def time_call(torch, fn, reps, prelude=None):
    """Mean / median / minimum of one call, each repetition bracketed by events; `prelude(i)` (untimed) runs before
    each repetition on the same stream, so that the call is measured in the state the path leaves the chip in."""
    for i in range(2):
        if prelude:
            prelude(i)
        fn(i)
    ms = []
    for i in range(reps):
        if prelude:
            prelude(i)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn(i)
        b.record()
        torch.cuda.synchronize()
        ms.append(a.elapsed_time(b))
    return stats(ms)


def layer_stack(torch, mk, cfg, n_layers, have, schedule):
    """The path over a whole stack of resident layers with immediate layer-by-layer eviction.  schedule = "device":
    per layer score -> maskkv_head_budgets (budgets stay on the device, k_l = the configuration's average) -> select
    -> compact into the layer's own cache -> attend.  schedule = "config": the configuration's per-layer budgets,
    known to the host and checked against the capacity by the call.  Timed eagerly and as one captured HIP graph;
    every graph replay is compared with the eager result."""
    from paper_2510_09309_amd import synth
    H, d, P, n_m = cfg["H"], cfg["d"], cfg["P"], cfg["n_m"]
    desc = mk.Desc(B=1, H=H, d=d, dtype=mk.MASKKV_BF16, n_resp=n_m, P_max=P)
    stride = (P + 63) // 64 * 64
    layers = list(have) + [device_layer(torch, cfg, l) for l in range(len(have), n_layers)]
    layers = layers[:n_layers]
    resp = [(mk.tensor_view(K, seq_start=[P]), mk.tensor_view(V, seq_start=[P])) for (_, K, V) in layers]
    dev = dict(device="cuda")
    alpha = 0.1
    if schedule == "device":
        host_budgets = [None] * n_layers
        caps = [H * cfg["budget_avg"]] * n_layers
        budgets = [torch.empty(H, dtype=torch.int32, **dev) for _ in layers]
    else:
        host_budgets = [synth.config_budgets(cfg["name"], l).tolist() for l in range(n_layers)]
        caps = [int(sum(b)) for b in host_budgets]
        budgets = [torch.tensor(b, dtype=torch.int32, **dev) for b in host_budgets]
    scores = torch.empty((H, stride), dtype=torch.float32, **dev)
    mass = [torch.empty(H, dtype=torch.float32, **dev) for _ in layers]
    idx = [torch.zeros(c, dtype=torch.int32, **dev) for c in caps]
    cu = [torch.empty(H + 1, dtype=torch.int32, **dev) for _ in layers]
    Kc = [torch.zeros((c, d), dtype=torch.bfloat16, **dev) for c in caps]
    Vc = [torch.zeros((c, d), dtype=torch.bfloat16, **dev) for c in caps]
    O = [torch.empty((1, H, n_m, d), dtype=torch.bfloat16, **dev) for _ in layers]
    ws = lambda n: torch.empty(max(n, 256), dtype=torch.uint8, **dev)
    ws_score, ws_sel = ws(mk.maskkv_score_workspace_bytes(desc)), ws(mk.maskkv_select_workspace_bytes(desc))
    ws_att = ws(mk.maskkv_attend_workspace_bytes(desc, False))

    def run_stack(stream):
        for l, (Q, K, V) in enumerate(layers):
            mk.maskkv_score(desc, Q, K, 0.0, scores, stride, mass[l], ws_score, stream)
            if schedule == "device":
                mk.maskkv_head_budgets(desc, mass[l], cfg["budget_avg"], alpha, budgets[l], stream)
            mk.maskkv_select(desc, scores, stride, cfg["window"], mk.POOL_MEAN, budgets[l], idx[l], cu[l], caps[l],
                             ws_sel, stream, budgets_host=host_budgets[l])
            mk.maskkv_compact(desc, K, V, idx[l], cu[l], caps[l], Kc[l], Vc[l], stream)
            mk.maskkv_attend(desc, Q, Kc[l], Vc[l], cu[l], caps[l], resp[l][0], resp[l][1], 0.0, O[l], None, ws_att,
                             stream)

    def timed(fn, reps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    cur = torch.cuda.current_stream()
    run_stack(cur)                      # warm-up (also the one-time kernel attribute calls)
    ms_eager = timed(lambda: run_stack(cur), 3)
    want = [(idx[l].clone(), O[l].clone()) for l in (0, n_layers - 1)]

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(cur)
    with torch.cuda.graph(graph, stream=side):
        run_stack(torch.cuda.current_stream())
    ok = True
    for _ in range(3):                  # replays with eager work and synchronisation in between
        for l in (0, n_layers - 1):
            idx[l].zero_()
            O[l].zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ok = ok and all(torch.equal(idx[l], w[0]) and torch.equal(O[l], w[1])
                        for l, w in zip((0, n_layers - 1), want))
    ms_graph = timed(graph.replay, 3)
    kept = [int(c[-1].item()) for c in cu]
    best = min(ms_eager, ms_graph)
    return {"workload": f"{cfg['name']}: {n_layers} resident layers, P={P}, {H} heads x {d}, {n_m} mask queries",
            "layers": n_layers, "ms_eager": ms_eager, "ms_graph": ms_graph, "ms_per_layer": best / n_layers,
            "graph_replays_match_eager": bool(ok),
            "prompt_tokens_per_s_whole_stack": P / (best * 1e-3),
            "prompt_tokens_per_s_per_layer": P * n_layers / (best * 1e-3),
            "budgets": (f"on-device head budgets, k_l={cfg['budget_avg']}, alpha={alpha}" if schedule == "device" else
                        f"the configuration's schedule: {caps[0] // H}/head at the first and last layer, "
                        f"{caps[1] // H}/head in between, 2:1 per-head split"),
            "kept_rows_per_layer_min_max": [min(kept), max(kept)], "capacity_per_layer_min_max": [min(caps), max(caps)]}


def batched_ragged(torch, mk, synth):
    """The batched ragged configuration: 8 sequences, prompts drawn in 4k..16k, 512 mask queries, per-head budgets
    log-uniform in 64..1024.  Compression once (score, select, compact over the ragged batch), then 64 denoising
    steps that each attend with fresh response Q/K/V over the fixed evicted cache.  This is the shape at which the
    gather moves enough bytes, and the attention enough flops, for a rate to mean something."""
    cfg = workload("C5")
    B, H, d, n_m, steps = cfg["B"], cfg["H"], cfg["d"], cfg["n_m"], cfg["steps"]
    P = [int(x) for x in synth.c5_prompt_lengths()]
    P_max = max(P)
    desc = mk.Desc(B=B, H=H, d=d, dtype=mk.MASKKV_BF16, n_resp=n_m, P_max=P_max, prompt_len=P)
    g = torch.Generator(device="cuda")
    g.manual_seed(cfg["seed"])
    sc = 1.0 / d ** 0.5
    dev = dict(device="cuda")

    def gauss(shape):
        return (torch.randn(shape, generator=g, dtype=torch.float32, **dev) * sc).to(torch.bfloat16)
    K, V, Q = gauss((B, H, P_max + n_m, d)), gauss((B, H, P_max + n_m, d)), gauss((B, H, n_m, d))
    u = torch.randn((B, H, d), generator=g, dtype=torch.float32, **dev)
    u = (u / u.norm(dim=2, keepdim=True)).to(torch.bfloat16)
    Q += u[:, :, None, :]                      # same recipe as device_layer: a direction per head shared by the
    for b in range(B):                         # mask queries and the planted fraction of the prompt keys
        for h in range(H):
            pos = torch.randperm(P[b], generator=g, device="cuda")[:round(cfg["planted_frac"] * P[b])]
            K[b, h, pos] += cfg["amplitude"] * u[b, h]
    fresh = [(gauss((B, H, n_m, d)), gauss((B, H, n_m, d)), gauss((B, H, n_m, d))) for _ in range(4)]
    bud_h = synth.config_budgets("C5")
    budgets = torch.from_numpy(bud_h).cuda()
    cap = int(bud_h.sum())
    stride = (P_max + 63) // 64 * 64
    scores = torch.empty((B * H, stride), dtype=torch.float32, **dev)
    mass = torch.empty(B * H, dtype=torch.float32, **dev)
    idx = torch.empty(cap, dtype=torch.int32, **dev)
    cu = torch.empty(B * H + 1, dtype=torch.int32, **dev)
    Kc = torch.empty((cap, d), dtype=torch.bfloat16, **dev)
    Vc = torch.empty_like(Kc)
    O = torch.empty((B, H, n_m, d), dtype=torch.bfloat16, **dev)
    ws = lambda n: torch.empty(max(n, 256), dtype=torch.uint8, **dev)
    w_sc, w_sel = ws(mk.maskkv_score_workspace_bytes(desc)), ws(mk.maskkv_select_workspace_bytes(desc))
    w_att = ws(mk.maskkv_attend_workspace_bytes(desc, False))
    bud_list = bud_h.tolist()

    score = lambda i: mk.maskkv_score(desc, Q, K, 0.0, scores, stride, mass, w_sc)
    select = lambda i: mk.maskkv_select(desc, scores, stride, cfg["window"], mk.POOL_MEAN, budgets, idx, cu, cap,
                                        w_sel, budgets_host=bud_list)
    compact = lambda i: mk.maskkv_compact(desc, K, V, idx, cu, cap, Kc, Vc)
    attend = lambda i: mk.maskkv_attend(desc, fresh[i % 4][0], Kc, Vc, cu, cap, fresh[i % 4][1], fresh[i % 4][2], 0.0,
                                        O, None, w_att)
    t_score = time_call(torch, score, 4)
    t_select = time_call(torch, select, 6, prelude=score)       # each measured right behind the call that precedes it
    t_compact = time_call(torch, compact, 6, prelude=lambda i: (score(i), select(i)))
    attend(0)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    a.record()
    for i in range(steps):
        attend(i)
    b.record()
    torch.cuda.synchronize()
    t_attend = a.elapsed_time(b) / steps
    flop_qk = 2.0 * n_m * d * H * sum(p + n_m for p in P)
    flop_att = 4.0 * n_m * d * (cap + B * H * n_m)
    evict_ms = t_score["median"] + t_select["median"] + t_compact["median"]
    gather_bytes = 2.0 * 2 * cap * d * 2
    return {"workload": f"C5: {B} sequences, prompts {min(P)}..{max(P)} (sum {sum(P)}), {H} heads x {d}, bf16, {n_m} mask "
                        f"queries, budgets {cfg['budget_lo']}..{cfg['budget_hi']} log-uniform ({cap} kept rows); "
                        f"{steps} denoising steps",
            "ms": {"score": t_score, "select": t_select, "compact": t_compact, "attend_per_step": t_attend},
            "prompt_tokens_scored_evicted_per_s": sum(P) / (evict_ms * 1e-3),
            "score_tflops_algorithmic": flop_qk / (t_score["median"] * 1e-3) / 1e12,
            "select_gbs": (4.0 * H * sum(P) + 4.0 * cap) / (t_select["median"] * 1e-3) / 1e9,
            "gather_gbs": gather_bytes / (t_compact["median"] * 1e-3) / 1e9,
            "gather_frac_of_hbm_peak": gather_bytes / (t_compact["median"] * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "attend_tflops": flop_att / (t_attend * 1e-3) / 1e12,
            "attend_frac_of_mfma_peak": flop_att / (t_attend * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
            "compress_once_plus_steps_ms": evict_ms + steps * t_attend}


def measured_peaks(torch, bb):
    """What this machine sustains on the resources that bound the kernels, from the probe kernels of the measurement
    library: bf16 MFMA issue from registers (on constant operands and on Gaussian bf16 data), v_exp_f32, streaming."""
    out = torch.empty(2048 * 256, dtype=torch.float32, device="cuda")
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").random_(0, 255)
    dst = torch.empty_like(src)
    g = torch.Generator(device="cuda")
    g.manual_seed(7)
    operands = (torch.randn(64 * 24 * 8, generator=g, device="cuda") / 128 ** 0.5).to(torch.bfloat16)  # like Q, K rows

    def rate(fn, reps):
        work = fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return work * reps / (a.elapsed_time(b) * 1e-3)
    mfma = rate(lambda: bb.maskkv_bench_probe(0, 20000, None, out, 512), 3)      # two waves per SIMD
    data2 = rate(lambda: bb.maskkv_bench_probe(5, 5000, operands, out, 512), 3)  # two waves per SIMD
    data1 = rate(lambda: bb.maskkv_bench_probe(5, 5000, operands, out, 256), 3)  # one wave per SIMD
    pipe2 = rate(lambda: bb.maskkv_bench_probe(6, 5000, operands, out, 512), 3)  # two waves per SIMD, as score pass 2
    pipe4 = rate(lambda: bb.maskkv_bench_probe(6, 5000, operands, out, 1024), 3) # four waves per SIMD
    exps = rate(lambda: bb.maskkv_bench_probe(1, 20000, None, out, 2048), 3)     # eight waves per SIMD
    mix = rate(lambda: bb.maskkv_bench_probe(4, 5000, None, out, 512), 3)        # two waves per SIMD, as score pass 2

    def ns_per_iteration(which, iters=5000):   # 256 eight-wave workgroups: one matrix wave + one vector wave per SIMD
        bb.maskkv_bench_probe(which, iters, operands, out, 256)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(3):
            bb.maskkv_bench_probe(which, iters, operands, out, 256)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e6 / (3 * iters)
    split = {"both_halves": ns_per_iteration(7), "matrix_waves_alone": ns_per_iteration(8),
             "vector_waves_alone": ns_per_iteration(9)}
    split["both_over_the_longer_alone"] = split["both_halves"] / max(split["matrix_waves_alone"],
                                                                       split["vector_waves_alone"])
    copy = rate(lambda: bb.maskkv_bench_probe(2, 0, src, dst, 2048), 5)
    read = rate(lambda: bb.maskkv_bench_probe(3, 0, src, out, 2048), 5)
    return {"mfma_bf16_tflops_constant_operands": mfma / 1e12,
            "mfma_bf16_tflops_gaussian_operands": {"two_waves_per_simd": data2 / 1e12, "one_wave_per_simd": data1 / 1e12},
            "v_exp_f32_per_s": exps, "stream_copy_gbs": copy / 1e9, "stream_read_gbs": read / 1e9,
            "score_instruction_mix_tflops": mix / 1e12,
            "score_pipeline_on_gaussian_operands_tflops": {"two_waves_per_simd": pipe2 / 1e12,
                                                           "four_waves_per_simd": pipe4 / 1e12},
            "matrix_and_vector_waves_on_one_simd_ns_per_iteration": split,
            "how": "maskkv_bench_probe: register-only v_mfma_f32_32x32x16_bf16 loops (constant operands; Gaussian bf16 "
                   "operands read once from memory into registers), v_exp_f32 loop on 2048 workgroups, 1 GiB copy "
                   "(read + written bytes), 1 GiB read; instruction mix = 16 MFMAs + 32 x (fma, exp, add) per lane per "
                   "iteration on 512 workgroups, no memory traffic; pipeline = the same sixteen MFMAs on Gaussian operands "
                   "into one accumulator pair while the exponentials consume the pair formed one iteration earlier; matrix and "
                   "vector waves = 256 eight-wave workgroups whose waves 0-3 issue those sixteen MFMAs and whose waves 4-7 "
                   "issue 32 x (multiply, exp, add) per iteration (waves w and w+4 share a SIMD), together and each half alone"}


def layer_importance_rate(torch, mk, n_tokens, hidden=4096):
    """Layer-importance reduction over [n_tokens, hidden] bf16 hidden states (LLaDA-8B's width): HBM-bound."""
    sets = []
    for i in range(2):  # two input sets (1.1 GB), so that no call finds its rows in a cache
        g = torch.Generator(device="cuda")
        g.manual_seed(900 + i)
        a = torch.randn((n_tokens, hidden), generator=g, device="cuda", dtype=torch.float32)
        b = a + 0.5 * torch.randn((n_tokens, hidden), generator=g, device="cuda", dtype=torch.float32)
        sets.append((a.to(torch.bfloat16), b.to(torch.bfloat16)))
        del a, b
    out = torch.empty(1, dtype=torch.float32, device="cuda")
    ws = torch.empty(mk.maskkv_layer_importance_workspace_bytes(), dtype=torch.uint8, device="cuda")
    for i in range(4):
        mk.maskkv_layer_importance(sets[i % 2][0], sets[i % 2][1], out, ws)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 16
    torch.cuda.synchronize()
    e0.record()
    for i in range(reps):
        mk.maskkv_layer_importance(sets[i % 2][0], sets[i % 2][1], out, ws)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    nbytes = 2.0 * n_tokens * hidden * 2
    return {"n_tokens": n_tokens, "hidden": hidden, "ms": ms, "bound": "hbm", "achieved_GBs": nbytes / (ms * 1e-3) / 1e9,
            "peak_GBs": HBM_PEAK_GBS, "frac": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "importance": float(out.item())}


def oracle_layer_seconds(cfg, budgets, budget_seconds, H_sample=4):
    """Seconds per layer of the float64 oracle (score + pool + select + compact + attend, head by head) on the host
    cores, from as many head passes of the configuration as fit in `budget_seconds` (at least one)."""
    from oracle import maskkv_oracle as orc
    from paper_2510_09309_amd import synth
    H_sample = min(H_sample, cfg["H"])
    L = synth.make_layer(cfg["seed"], H=H_sample, d=cfg["d"], P=cfg["P"], n_m=cfg["n_m"], dtype=cfg["dtype"],
                         n_planted=cfg["n_planted"], amplitude=cfg["amplitude"])
    done, t0 = 0, time.perf_counter()
    while True:
        h = done % H_sample
        I, _ = orc.score(L.Q[h], L.K[h], L.P)
        keep = orc.select(orc.pool(I, cfg["window"]), int(budgets[done % cfg["H"]]))
        Kc, Vc = orc.compact(L.K[h, :L.P], L.V[h, :L.P], keep)
        orc.attend(L.Q[h], Kc, Vc, L.K[h, L.P:], L.V[h, L.P:])
        done += 1
        el = time.perf_counter() - t0
        if el >= budget_seconds:
            break
    return el / done * cfg["H"], done, el


def cpu_oracle_baseline(cfg, budget_seconds=12.0):
    """The oracle as it stands, timed on the host: ~12 s of head passes of the benchmarked workload, then short
    samples of the other configurations (per-layer and per-stack figures are extrapolated from the sampled heads)."""
    import torch
    from oracle import maskkv_oracle as orc
    from paper_2510_09309_amd import synth
    per_layer, done, el = oracle_layer_seconds(cfg, synth.config_budgets(cfg["name"]), budget_seconds)
    others = {}
    for name, secs in (("C1", 0.5), ("C2", 2.0), ("C3", 2.0)):
        c = workload(name)
        s_layer, n, t = oracle_layer_seconds(c, synth.config_budgets(name), secs)
        others[name] = {"s_per_layer": s_layer, "prompt_tokens_per_s_per_layer": c["P"] / s_layer,
                        "sample": f"{n} head passes of one layer ({c['H']} heads) in {t:.1f} s" +
                                  (f"; x{c['layers']} layers = {s_layer * c['layers']:.1f} s extrapolated"
                                   if c["layers"] > 1 else "")}
    # batched ragged configuration: compression of two (sequence, head) pairs and three denoising steps on each
    c5 = workload("C5")
    lens = synth.c5_prompt_lengths(c5)
    bud = synth.config_budgets("C5")
    t0 = time.perf_counter()
    pairs, t_steps = 0, 0.0
    for b in sorted({int(np.argmin(lens)), int(np.argmax(lens))}):
        L = synth.config_layer("C5", b=b)
        I, _ = orc.score(L.Q[0], L.K[0], L.P)
        keep = orc.select(orc.pool(I, c5["window"]), int(bud[b * c5["H"]]))
        Kc, Vc = orc.compact(L.K[0, :L.P], L.V[0, :L.P], keep)
        pairs += 1
        t1 = time.perf_counter()
        for step in range(3):
            Qs, Ks, Vs = synth.make_response_step(c5["seed"] + 1 + step, 1, c5["d"], c5["n_m"], "bf16")
            orc.attend(Qs[0], Kc, Vc, Ks[0], Vs[0])
        t_steps += time.perf_counter() - t1
    t_c5 = time.perf_counter() - t0
    t_compress = (t_c5 - t_steps) / pairs          # includes drawing the inputs of the pair
    t_step = t_steps / (3 * pairs)
    others["C5"] = {"s_compress_per_sequence_head": t_compress, "s_per_attend_step_per_sequence_head": t_step,
                    "s_compress_plus_steps_extrapolated": (t_compress + c5["steps"] * t_step) * c5["B"] * c5["H"],
                    "sample": f"{pairs} (sequence, head) pairs (shortest and longest prompt, head 0): input draw + "
                              f"compression + 3 steps each in {t_c5:.1f} s; x{c5['B'] * c5['H']} pairs and "
                              f"{c5['steps']} steps extrapolated"}
    return {
        "value": cfg["P"] / per_layer, "unit": "prompt tokens/s per layer (score+select+compact+attend)",
        "cores": int(torch.get_num_threads()), "kind": "oracle",
        "sample": f"{done} head passes (score+pool+select+compact+attend, float64 numpy) of the same workload in "
                  f"{el:.1f} s; one layer = {cfg['H']} heads -> {per_layer:.2f} s/layer",
        "host_cpu_count": os.cpu_count(), "other_configurations": others,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="C4", choices=["C2", "C3", "C4"])
    ap.add_argument("--resident-layers", type=int, default=4)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--stack-layers", type=int, default=32,
                    help="after the timed region, also run whole stacks of this many resident layers (the workload "
                         "with on-device head budgets and the 8k-prompt configuration with its budget schedule), "
                         "eagerly and as one HIP graph; 0 skips them")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip what runs after the timed region besides the full-cache attention: peaky logits, the "
                         "4k-prompt layer, the 8k-prompt stack, the batched ragged configuration, layer importance "
                         "and the probes")
    ap.add_argument("--batched-only", action="store_true",
                    help="run only the batched ragged configuration and print its block (for profiling that shape on "
                         "its own; this is not the benchmark line)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="before the warm-up, copy 256 MiB device-to-device three times: a kernel of known traffic "
                         "against which rocprofv3's FETCH_SIZE / WRITE_SIZE counters are scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures the hot path on ONE GPU; --gpus must be 1 (the path is independent per "
              "head and would shard over heads or sequences without any collective)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2510_09309_amd import bench_binding as bb, binding as mk, synth

    torch.cuda.set_device(0)

    def calibration_copy():
        src = torch.empty(256 * 1024 * 1024, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    if args.batched_only:
        if args.calibration_copy:
            calibration_copy()
        print(json.dumps({"batched": batched_ragged(torch, mk, synth)}))
        return

    cfg = workload(args.workload)
    H, d, P, n_m = cfg["H"], cfg["d"], cfg["P"], cfg["n_m"]
    N = P + n_m
    budgets_h = synth.config_budgets(args.workload, layer=1)      # the schedule's interior layers
    cap = int(budgets_h.sum())
    budgets = torch.from_numpy(budgets_h).cuda()
    layers = [device_layer(torch, cfg, l) for l in range(args.resident_layers)]
    path = Path(torch, mk, cfg, layers, cap)
    hev = HipEvents()
    stream = torch.cuda.current_stream()

    if args.calibration_copy:
        calibration_copy()

    # ---- the timed region: exactly --steps whole-path steps
    tr = timed_steps(torch, hev, path, budgets, args.steps, args.warmup, bb)
    ms_per_step = tr["wall_ms_per_step"]
    pass1_ms = float(np.mean(tr["pass1"]))
    evict_ms = float(np.mean(tr["evict"]))
    attend_ms = float(np.mean(tr["attend"]))
    # ---- the same steps again with every call bracketed (each extra event costs the step a few microseconds)
    tb = timed_steps(torch, hev, path, budgets, max(16, args.steps // 2), 2, bb, every_call=True)
    score_ms = float(np.mean(tb["score"]))
    compact_ms = float(np.mean(tb["compact"]))

    # ---- the un-evicted attention (what the eviction removes), each call behind a compressed one as in the path
    reps = max(4, args.steps // 8)
    t_full = time_call(torch, lambda i: path.attend_full(i, stream), reps, prelude=lambda i: path.attend(i, stream))
    t_score_hot = time_call(torch, lambda i: path.score(0, stream), reps)

    keys_compressed = cap + H * n_m
    flop_attend = 4.0 * n_m * d * keys_compressed
    flop_full = 4.0 * n_m * d * N * H
    flop_qk_all = 2.0 * n_m * d * N * H              # one QK^T over all keys: the method's scoring work
    bytes_k = 2.0 * N * d * H                        # K read once, bf16
    bytes_gather = 2.0 * 2 * cap * d * 2             # K and V rows, read + write

    out = {
        "metric": "prompt tokens scored+evicted/s per layer; compressed-attn TFLOP/s @32k prompt",
        "value": P / (evict_ms * 1e-3),
        "unit": "prompt tokens/s per layer = P / (score + select + compact), all heads: the interval from the start of a "
                "step to the end of its compact, between HIP events in the timed region",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: 1 sequence, {H} heads x {d}, bf16, P={P}, {n_m} mask queries, "
                               f"budget {cap // H}/head avg (2:1 split), pool window {cfg['window']}; one layer per "
                               f"step (score, select, compact, attend), {len(layers)} resident layers rotated",
                   "global_batch": 1, "seq_len": N},
        "whole_step_prompt_tokens_per_s": P / (ms_per_step * 1e-3),
        "timed_region_ms": {k: stats(tr[k]) for k in ("evict", "pass1", "attend", "step")},
        "every_call_bracketed_ms": {"steps": len(tb["step"]), "ms_per_step": tb["wall_ms_per_step"],
                                    **{k: stats(tb[k]) for k in ("score", "pass1", "select", "compact", "attend",
                                                                 "evict", "step")}},
        "breakdown_ms": {"score": score_ms, "select": float(np.mean(tb["select"])), "compact": compact_ms,
                         "attend": float(np.mean(tb["attend"])), "attend_full": t_full["median"],
                         "score_pass1_in_timed_region": pass1_ms, "score_hot_same_layer": t_score_hot["median"]},
        "attend_full_ms": t_full,
        "attend_compressed_tflops": flop_attend / (attend_ms * 1e-3) / 1e12,
        "attend_compressed_frac_of_mfma_peak": flop_attend / (attend_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
        "attend_full_tflops": flop_full / (t_full["median"] * 1e-3) / 1e12,
        "attend_full_frac_of_mfma_peak": flop_full / (t_full["median"] * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
        "attend_speedup_full_over_compressed": t_full["median"] / attend_ms,
        "attend_flop_ratio_full_over_compressed": flop_full / flop_attend,
        "score_k_read_gbs_algorithmic": bytes_k / (score_ms * 1e-3) / 1e9,
        "gather_gbs": bytes_gather / (compact_ms * 1e-3) / 1e9,
        "roofline": {
            "kernel": "score_kernel<bf16,128,pass 1> (QK^T over all keys + exp + row statistics)",
            "bound": "mfma", "achieved": flop_qk_all / (pass1_ms * 1e-3) / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS,
            "unit": "TFLOP/s", "frac": flop_qk_all / (pass1_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
            "traffic": SCORE_PASS1_TRAFFIC_BYTES.get(args.workload),
            "note": "achieved = the method's one QK^T (2*n_m*N*d*H flop) over the duration of pass 1 alone; maskkv_score "
                    "forms the logits twice (pass 1, merge, pass 2): whole_call prices the call on the same single QK^T",
            "whole_call": {"what": "maskkv_score (pass 1 + merge + pass 2)",
                           "achieved": flop_qk_all / (score_ms * 1e-3) / 1e12,
                           "frac": flop_qk_all / (score_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                           "frac_counting_executed_flops":
                               2.0 * flop_qk_all / (score_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS},
            "hbm_view": {"achieved_GBs": (bytes_k + 2.0 * n_m * d * H) / (pass1_ms * 1e-3) / 1e9,
                         "peak_GBs": HBM_PEAK_GBS},
        },
    }

    if not args.no_extras:
        # ---- scoring when the rows' normalisers come from the model's own first-step attention over the full sequence
        # (maskkv_attend_full returns them): the second scoring pass alone.  Not the headline: `value` above is the
        # stand-alone two-pass call.
        path.row_lse = []
        for (Q, K, V) in layers:
            lse = torch.empty(H * n_m, dtype=torch.float32, device="cuda")
            mk.maskkv_attend_full(path.desc, Q, K, V, 0.0, path.Of, lse, path.ws_full, stream)
            path.row_lse.append(lse)
        tg = timed_steps(torch, hev, path, budgets, 32, 4, bb, every_call=True)
        path.row_lse = None
        out["given_row_lse"] = {
            "what": "the same step with maskkv_score_given_lse (row normalisers from maskkv_attend_full of the same "
                    "queries) in place of maskkv_score: 32 timed steps, every call bracketed by HIP events",
            "ms_per_step": tg["wall_ms_per_step"],
            "timed_region_ms": {k: stats(tg[k]) for k in ("score", "select", "compact", "attend", "evict")},
            "prompt_tokens_scored_evicted_per_s": P / (float(np.mean(tg["evict"])) * 1e-3)}
        # ---- the same MFMA calls on peaky logits (components 9.5 x wider: softmax rows concentrate on few keys, so
        # the lazily raised running references of scoring and attention leave their cheapest branch)
        peaky = [device_layer(torch, cfg, 100 + l, sigma=9.5) for l in range(2)]
        pk = Path(torch, mk, cfg, peaky, cap)
        pk.score(0, stream)
        pk.select(0, budgets, stream)
        pk.compact(0, stream)
        out["peaky_logits_ms"] = {
            "recipe": "Q, K, V components N(0,1)*9.5/sqrt(d) instead of N(0,1)/sqrt(d), same planting",
            "score": time_call(torch, lambda i: pk.score(i, stream), 8),
            "attend": time_call(torch, lambda i: pk.attend(i, stream), 8, prelude=lambda i: pk.compact(i, stream)),
            "attend_full": time_call(torch, lambda i: pk.attend_full(i, stream), 4)}
        del peaky, pk
        if args.workload != "C2":
            c2 = workload("C2")
            b2h = synth.config_budgets("C2")
            p2 = Path(torch, mk, c2, [device_layer(torch, c2, l) for l in range(4)], int(b2h.sum()))
            t2 = timed_steps(torch, hev, p2, torch.from_numpy(b2h).cuda(), 32, 4, bb, every_call=True)
            out["single_layer_4k_prompt"] = {
                "workload": f"C2: {c2['H']} heads x {c2['d']}, bf16, P={c2['P']}, {c2['n_m']} mask queries, budget "
                            f"{c2['budget_avg']}/head avg (2:1 split)",
                "ms_per_step": t2["wall_ms_per_step"],
                "timed_region_ms": {k: stats(t2[k]) for k in ("score", "select", "compact", "attend", "evict")},
                "prompt_tokens_scored_evicted_per_s": c2["P"] / (float(np.mean(t2["evict"])) * 1e-3)}
            del p2
    if args.stack_layers > 0:
        out["stack"] = layer_stack(torch, mk, cfg, args.stack_layers, layers, "device")
    del path, layers
    if args.stack_layers > 0 and not args.no_extras and args.workload != "C3":
        out["stack_8k_prompt"] = layer_stack(torch, mk, workload("C3"), args.stack_layers, [], "config")
    if not args.no_extras:
        out["layer_importance"] = layer_importance_rate(torch, mk, N)
        peaks = measured_peaks(torch, bb)
        n_exp = float(n_m) * N * H                       # exponentials of one pass
        gauss2 = peaks["mfma_bf16_tflops_gaussian_operands"]["two_waves_per_simd"]
        peaks["score_pass1_vs_measured"] = {
            "frac_of_mfma_on_constant_operands": out["roofline"]["achieved"] / peaks["mfma_bf16_tflops_constant_operands"],
            "frac_of_mfma_on_gaussian_operands": out["roofline"]["achieved"] / gauss2,
            "mfma_time_us_on_gaussian_operands": flop_qk_all / (gauss2 * 1e12) * 1e6,
            "exp_time_us": n_exp / peaks["v_exp_f32_per_s"] * 1e6,
            "instruction_mix_time_us": flop_qk_all / (peaks["score_instruction_mix_tflops"] * 1e12) * 1e6,
            "pipeline_on_gaussian_operands_time_us": flop_qk_all / (
                peaks["score_pipeline_on_gaussian_operands_tflops"]["two_waves_per_simd"] * 1e12) * 1e6,
            "k_stream_time_us": bytes_k / (peaks["stream_read_gbs"] * 1e9) * 1e6,
            "measured_us": pass1_ms * 1e3}
        out["measured_peaks"] = peaks
        out["batched"] = batched_ragged(torch, mk, synth)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_oracle_baseline(cfg)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
