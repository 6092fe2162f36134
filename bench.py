#!/usr/bin/env python3
"""Benchmark of the routed low-rank linear hot path on ONE MI355X.

A "step" is one pass of the whole prefill hot path over one batch of the q_proj-shaped workload
(bf16, 4096x4096, stored rank 2048 in 16 groups of 128, top-8, 8 prompts x 512 tokens):
  pool + route -> pattern-cache probe (route-on-miss) -> bucket -> pack (memory aggregation) -> fused forward.
All inputs are resident in HBM before the timed region.  `value` is whole-step prefill throughput in
TFLOP/s of algorithmic work 2*T*r_S*(n+m).  The `roofline` object prices the dominant kernel (the fused
forward) against the bf16 matrix-core peak from HIP-event timings taken inside the timed region; the
`decode` object reports the bandwidth-bound decode kernels on the MLP-shaped workload (32 sequences, 20
groups of 128, top-10, 4 patterns) against the HBM peak; `cpu_baseline` is the CPU oracle timed on the host.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline] [--no-decode] [--tokens T]
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 matrix-core peak
HBM_PEAK_GBS = 8000.0            # MI355X HBM3E peak


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--tokens", type=int, default=512, help="tokens per prompt (512 = the named workload)")
    ap.add_argument("--prompts", type=int, default=8)
    ap.add_argument("--decode-steps", type=int, default=128)
    ap.add_argument("--decode-copies", type=int, default=32, help="independent layer copies rotated per step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--only-decode", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the timed steps: skip the side records (other schedules, multi-layer calls, shared "
                         "head, rank-granular mode) so that a profile of the run holds the timed kernels alone")
    ap.add_argument("--stack", action="store_true",
                    help="also time the full 32-layer x 7-projection stack (prefill 1 x 2048 tokens, then decode steps)")
    ap.add_argument("--stack-decode-steps", type=int, default=256, help="decode steps timed after the prefill (the workload names 256)")
    ap.add_argument("--stress", action="store_true",
                    help="also run the pattern-cache / grouped-execution stress (256 ragged prompts, MLP-shaped layers)")
    ap.add_argument("--only-stress", action="store_true")
    ap.add_argument("--no-peaks", action="store_true", help="skip the achievable-peak probes")
    ap.add_argument("--only-peaks", action="store_true")
    ap.add_argument("--no-token-scaled", action="store_true", help="skip the 8 x 4096-token side record")
    ap.add_argument("--no-decode-graph", action="store_true", help="skip the HIP-graph replay of the decode steps")
    ap.add_argument("--no-prefill-graph", action="store_true",
                    help="time the prefill steps as eager launches only (the default also replays them from a HIP graph)")
    ap.add_argument("--no-decode-separate", action="store_true",
                    help="skip the comparison run that calls gate and up separately (counter runs use this)")
    return ap.parse_args()


def traffic_from_profiles(name):
    """HBM bytes per launch of the dominant kernel as measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE,
    scaled by a copy kernel of known size); the figure is kept in profiles/traffic.json by hand after a
    counter run, null until then."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as f:
            return json.load(f).get(name)
    except Exception:
        return None


def bench_prefill(args, torch, pa, si):
    from helpers import i32, upload_layer, upload_tokens
    dev = "cuda"
    w = si.config1(P=args.prompts, T=args.tokens)
    lay = w.layers[0]
    k, P, n, m, gs = w.k, w.P, lay.n, lay.m, lay.gs
    rS = k * gs
    rows = int(w.tok_offsets[-1])
    dl_rm = upload_layer(lay, dev)                         # row-major store (rank-granular aggregation reads it)
    dl = pa.layer_to_mfma16(dl_rm)
    X = upload_tokens(w.X, "bf16", dev)
    off = i32(w.tok_offsets, dev)
    Wr = torch.from_numpy(w.Wr).to(dev)                    # [1][G][d]
    n_slots = 32                                           # aggregated-pattern store, one slot per cache entry
    cache = pa.Cache(n_slots, w.d, 1, k, max(P, 8))
    # every buffer of the step is allocated once, outside the timed region
    emb = torch.empty((P, w.d), dtype=torch.float32, device=dev)
    sub_route = torch.empty((P, k), dtype=torch.int32, device=dev)
    ws_route = torch.empty(max(pa.route_workspace_bytes(rows, P, w.d), 256), dtype=torch.uint8, device=dev)
    entry = torch.empty(P, dtype=torch.int32, device=dev)
    hit = torch.empty(P, dtype=torch.uint8, device=dev)
    sim = torch.empty(P, dtype=torch.float32, device=dev)
    sub = torch.empty((P, 1, k), dtype=torch.int32, device=dev)
    bucket_out = (torch.empty(P, dtype=torch.int32, device=dev), torch.empty(P, dtype=torch.int32, device=dev),
                  torch.empty(P + 1, dtype=torch.int32, device=dev), torch.empty(1, dtype=torch.int32, device=dev),
                  torch.empty(P, dtype=torch.int32, device=dev))
    Vs = torch.empty((n_slots, rS, n), dtype=torch.bfloat16, device=dev)
    Us = torch.empty((n_slots, rS, m), dtype=torch.bfloat16, device=dev)
    Y = torch.empty((rows, m), dtype=torch.bfloat16, device=dev)
    ws_fwd = torch.empty(max(pa.lowrank_workspace_bytes(pa.PARSE_PREFILL, dl, rows, k, P, n_slots), 256), dtype=torch.uint8, device=dev)
    pt = pa.Patterns(k, n_slots, Vs, Us)
    plan = torch.empty(pa.prefill_plan_bytes(rows, P, n_slots), dtype=torch.uint8, device=dev)
    ws_plan = torch.empty(max(pa.lowrank_prefill_planned_workspace_bytes(dl, rows, P, k, n_slots), 256), dtype=torch.uint8, device=dev)
    names = ["pool", "cache", "bucket+plan", "pack", "forward"]

    def step(ev=None):
        def mark(i):
            if ev is not None:
                ev[i].record()
        mark(0)
        pa.pool(X, off, emb, ws_route)                      # the prompt embeddings; the router runs inside the probe, on a miss
        mark(1)
        cache.lookup_or_route(emb, 0.9, Wr, entry, hit, sim, sub)
        mark(2)
        # buckets of equal subsets (execution grouping) and the plan (token rows grouped by pattern = cache entry; it
        # serves every layer) come out of one launch
        pa.bucket_and_plan(sub, k, k, off, entry, rows, n_slots, bucket_out, plan)
        mark(3)
        pa.pack_new_entries(dl, sub, k, k, entry, hit, Vs, Us)   # aggregation happens once per new cache entry
        mark(4)
        pa.lowrank_prefill_planned(dl, pt, X, off, entry, plan, Y, ws_plan)   # two launches over the plan
        mark(5)

    # cold step: empty cache, every prompt misses, is routed, appended and aggregated
    step(); torch.cuda.synchronize()
    cache.clear()
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record(); step(); c1.record(); torch.cuda.synchronize()
    cold_ms = c0.elapsed_time(c1)
    assert int(hit.sum().item()) == 0 and cache.count() == P
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(evs[s])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    wall = t1 - t0
    per = {nm: sum(evs[s][i].elapsed_time(evs[s][i + 1]) for s in range(args.steps)) / args.steps * 1e3
           for i, nm in enumerate(names)}                                  # microseconds
    hits = int(hit.sum().item())
    # The same steps replayed from a HIP graph of consecutive steps (every launch of every step is a kernel node;
    # the library records no memset).  An even number of steps per graph (ten, or two when K is no multiple of ten),
    # because the cache probe alternates between two device counters from call to call; the probe grid is sized for the cache's capacity once the host-side bound has
    # reached it (it has, after the warm-up), so the recorded launches stay valid whatever the cache holds.
    # The eager loop above gives the per-row breakdown; K steps are timed again here as K/10 (K/2) replays.
    # (One linear chain of kernel nodes: putting bucket / pack / plan on parallel branches was measured slower, 148 us
    # per step against 127 -- dependencies across queues cost more than the three small kernels they would overlap.)
    graph = None
    if not args.no_prefill_graph and args.steps >= 2:
        Y_ref, entry_ref, hit_ref = Y.clone(), entry.clone(), hit.clone()
        spg = 10 if args.steps % 10 == 0 else 2      # an even number of steps per graph (the two counters)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(spg):
                step()
        for _ in range(2):
            g.replay()
        torch.cuda.synchronize()
        reps = args.steps // spg
        tg0 = time.perf_counter()
        for _ in range(reps):
            g.replay()
        torch.cuda.synchronize()
        tg1 = time.perf_counter()
        same = bool(torch.equal(Y.view(torch.int16), Y_ref.view(torch.int16)) and torch.equal(entry, entry_ref)
                    and torch.equal(hit, hit_ref))
        graph = {"ms_per_step": (tg1 - tg0) / (spg * reps) * 1e3, "steps": spg * reps, "steps_per_graph": spg,
                 "matches_eager_bitwise": same}
    sched_us, rank_us, pipelined = {}, None, None
    if not args.no_extras:
        # the same forward under each fixed schedule, for the record (not part of the timed steps above)
        pid = entry
        for nm, code in (("fused", pa.PARSE_SCHED_FUSED), ("tiles_two_launch", pa.PARSE_SCHED_TILES),
                         ("planned_incl_plan_launch", pa.PARSE_SCHED_PLANNED)):
            pts = pt.with_schedule(code)
            for _ in range(3):
                pa.lowrank_forward(pa.PARSE_PREFILL, dl, pts, X, off, pid, Y, ws_fwd)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(20):
                pa.lowrank_forward(pa.PARSE_PREFILL, dl, pts, X, off, pid, Y, ws_fwd)
            e1.record(); torch.cuda.synchronize()
            sched_us[nm] = round(e0.elapsed_time(e1) / 20 * 1e3, 2)
        # horizontal fusion, for the record: two layers of this shape that share X, in one call vs two calls
        # (the same factors stand in for the second layer; its output and intermediate are its own)
        Y2 = torch.empty_like(Y)
        ws2 = torch.empty(2 * ws_fwd.numel(), dtype=torch.uint8, device=dev)
        def timed(fn, reps=20):
            for _ in range(3):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                fn()
            e1.record(); torch.cuda.synchronize()
            return round(e0.elapsed_time(e1) / reps * 1e3, 2)
        sched_us["two_layers_one_call"] = timed(lambda: pa.lowrank_prefill_multi([dl, dl], [pt, pt], X, off, pid, [Y, Y2], ws2))
        sched_us["two_layers_two_calls"] = timed(lambda: (pa.lowrank_forward(pa.PARSE_PREFILL, dl, pt, X, off, pid, Y, ws_fwd),
                                                          pa.lowrank_forward(pa.PARSE_PREFILL, dl, pt, X, off, pid, Y2, ws_fwd)))
        # shared head, for the record (timing only: groups 0,1 stand in as the shared block, the per-pattern blocks
        # hold each prompt's last k-2 groups; parity of this layout is covered by the tests)
        ns = 2
        Vsh, Ush = pa.pack_experts(dl, torch.arange(ns, dtype=torch.int32, device=dev))
        Vp, Up = pa.pack_patterns(dl, sub.view(P, k)[:, ns:], k, k - ns, None, None, P)
        pt_sh = pa.Patterns(k, P, Vp, Up, Vt_shared=Vsh, Ut_shared=Ush, n_shared=ns)
        pid_seq = torch.arange(P, dtype=torch.int32, device=dev)
        sched_us["shared_head_2_of_8"] = timed(lambda: pa.lowrank_forward(pa.PARSE_PREFILL, dl, pt_sh, X, off, pid_seq, Y, ws_fwd))
        # rank-granular mode, for the record (the paper's own formulation: a router over all R ranks, top-K ranks,
        # K scattered rank rows aggregated per prompt); the forward then runs on blocks of the same shape as above
        K_r = rS
        Wr_r = torch.randn((lay.R, w.d), device=dev) / 64.0
        sub_r = torch.empty((P, K_r), dtype=torch.int32, device=dev)
        ws_r = torch.empty(int(pa.lib().parse_route_ranks_workspace_bytes(rows, P, w.d, lay.R)), dtype=torch.uint8, device=dev)
        Vr = torch.empty((P, K_r, n), dtype=torch.bfloat16, device=dev); Ur = torch.empty((P, K_r, m), dtype=torch.bfloat16, device=dev)
        rank_us = {"route_ranks": timed(lambda: pa.route_ranks(X, off, Wr_r, K_r, subset_out=sub_r, workspace=ws_r)),
                   "pack_ranks_8_patterns": timed(lambda: pa.pack_ranks(dl_rm, sub_r, K_r, P, Vt_S=Vr, Ut_S=Ur)),
                   "R": lay.R, "K": K_r}
        # two batches in flight, for the record: the control path (pool+route, cache, bucket, pack) of batch i+1 runs
        # on a second stream while batch i's forward runs; per-batch buffers are double-buffered, events order the
        # two streams (default priorities).  Every batch still does every row of the path; only the throughput of a
        # stream of batches changes, a single batch's latency does not.
        bufs = []
        for _ in range(2):
            bufs.append(dict(emb=torch.empty_like(emb), sub_route=torch.empty_like(sub_route), entry=torch.empty_like(entry),
                             hit=torch.empty_like(hit), sim=torch.empty_like(sim), sub=torch.empty_like(sub),
                             bucket=tuple(torch.empty_like(t) for t in bucket_out), Y=torch.empty_like(Y),
                             plan=torch.empty_like(plan),
                             ready=torch.cuda.Event(), done=torch.cuda.Event()))
        s_ctl, s_fwd = torch.cuda.Stream(), torch.cuda.Stream()
        ws_route2 = torch.empty_like(ws_route)
        def run_pipelined(n_batches):
            for i in range(n_batches):
                b = bufs[i & 1]
                with torch.cuda.stream(s_ctl):
                    if i >= 2:
                        s_ctl.wait_event(b["done"])            # batch i-2 has finished reading this buffer set
                    pa.pool(X, off, b["emb"], ws_route2)
                    cache.lookup_or_route(b["emb"], 0.9, Wr, b["entry"], b["hit"], b["sim"], b["sub"])
                    pa.bucket_and_plan(b["sub"], k, k, off, b["entry"], rows, n_slots, b["bucket"], b["plan"])
                    pa.pack_new_entries(dl, b["sub"], k, k, b["entry"], b["hit"], Vs, Us)
                    b["ready"].record(s_ctl)
                with torch.cuda.stream(s_fwd):
                    s_fwd.wait_event(b["ready"])
                    pa.lowrank_prefill_planned(dl, pt, X, off, b["entry"], b["plan"], b["Y"], ws_plan)
                    b["done"].record(s_fwd)
        torch.cuda.synchronize()
        run_pipelined(6); torch.cuda.synchronize()
        nb = max(args.steps, 10)
        tp0 = time.perf_counter(); run_pipelined(nb); torch.cuda.synchronize(); tp1 = time.perf_counter()
        pa.lowrank_prefill_planned(dl, pt, X, off, entry, plan, Y, ws_plan); torch.cuda.synchronize()
        pipelined = {"batches": nb, "ms_per_batch": round((tp1 - tp0) / nb * 1e3, 4),
                     "TFLOPs": round(2.0 * rows * rS * (n + m) / ((tp1 - tp0) / nb) / 1e12, 1),
                     "same_output_as_sequential": bool(torch.equal(bufs[0]["Y"], Y) and torch.equal(bufs[1]["Y"], Y))}
        # router training step, for the record (Sec. 4.2): loss and gradient of Wr for this batch against a random
        # "dense" target; two full-rank products (137 GFLOP) plus small reductions
        scores_t = torch.empty((P, lay.G), dtype=torch.float32, device=dev)
        pa.route(X, off, Wr[0], k, subset_out=sub_route, scores_out=scores_t, emb_out=emb, workspace=ws_route)
        Yd_t = torch.randn((rows, m), device=dev).to(torch.bfloat16)
        Utr = pa.rankmajor_left_factor(dl_rm)
        ws_t = torch.empty(int(pa.lib().parse_router_grad_workspace_bytes(C.byref(dl.c()), rows, P)), dtype=torch.uint8, device=dev)
        sched_us["router_training_step"] = timed(lambda: pa.router_grad(dl, Utr, X, off, Y, Yd_t, emb, scores_t, k, 1.0, 1e-6, ws_t))
    pa.route(X, off, Wr[0], k, subset_out=sub_route, workspace=ws_route); torch.cuda.synchronize()
    assert torch.equal(sub.view(P, k), sub_route), "cache answered with a subset that differs from the route"
    flops = 2.0 * rows * rS * (n + m)
    eager_ms = wall / args.steps * 1e3
    use_graph = graph is not None and graph["matches_eager_bitwise"] and graph["steps"] == args.steps
    ms_per_step = graph["ms_per_step"] if use_graph else eager_ms
    value = flops / (ms_per_step * 1e-3) / 1e12
    fwd_s = per["forward"] * 1e-6
    achieved = flops / fwd_s / 1e12
    cache.close()
    res = {
        "value": value, "ms_per_step": ms_per_step, "flops_per_step": flops,
        "launch_mode": "graph" if use_graph else "eager", "eager_ms_per_step": eager_ms,
        "graph_replay": None if graph is None else {**graph, "ms_per_step": round(graph["ms_per_step"], 4)},
        "rows_us": {k_: round(v, 2) for k_, v in per.items()},
        "cache_hits": hits, "forward_us_by_schedule": sched_us, "cold_step_ms": round(cold_ms, 4),
        "rank_granular_us": rank_us, "two_batches_in_flight": pipelined,
        # the forward of the timed steps is parse_lowrank_prefill_planned: both products on LDS-staged tiles over the
        # plan, 128 x 128 for the first (256 workgroups), 256 x 256 for the second
        "roofline": {"bound": "mfma", "kernel": "gemm_lds<128,128,2x2,BK64,S4> + gemm_lds<256,256,2x4,BK32,S4> (one planned forward call)",
                     "achieved": round(achieved, 2),
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4),
                     "traffic": traffic_from_profiles("prefill_config1"),
                     "launch_us": round(per["forward"], 2)},
        "workload": w,
    }
    return res


def bench_decode(args, torch, pa, si):
    """MLP-shaped decode: gate/up (4096->11008) and down (11008->4096), R=2560 in 20 groups, top-10, 32
    sequences, 4 patterns.  `copies` independent layer triples are rotated so that every step streams cold
    factors from HBM (one triple is about the size of the last-level cache).  Factor values are Gaussian
    (their layout is irrelevant to timing); parity at these shapes is covered by the tests."""
    import numpy as np
    dev = "cuda"
    B, G, k, R, hidden, inter = 32, 20, 10, 2560, 4096, 11008
    gs = R // G
    shapes = [("gate", hidden, inter), ("up", hidden, inter), ("down", inter, hidden)]
    rng = np.random.default_rng(si.SEED_BASE + 2)
    pats = np.stack([np.sort(rng.choice(G, size=k, replace=False)) for _ in range(4)]).astype(np.int32)
    distinct = len(set(pats.reshape(-1).tolist()))
    seq_pat = (np.arange(B) % 4).astype(np.int32)
    subsets = torch.from_numpy(pats).to(dev)
    pid = torch.from_numpy(seq_pat).to(dev)
    copies = args.decode_copies
    layers = []
    for c in range(copies):
        trip = []
        for nm, n, m in shapes:
            Vt = (torch.randn((R, n), device=dev) * 0.02).to(torch.bfloat16)
            Ut = (torch.randn((R, m), device=dev) * 0.02).to(torch.bfloat16)
            trip.append(pa.Layer(Vt, Ut, n, m, R, G, pa.PARSE_MFMA16))
        layers.append(trip)
    xs = {hidden: torch.randn((B, hidden), device=dev).to(torch.bfloat16),
          inter: torch.randn((B, inter), device=dev).to(torch.bfloat16)}
    ys = {hidden: torch.empty((B, hidden), dtype=torch.bfloat16, device=dev),
          inter: torch.empty((B, inter), dtype=torch.bfloat16, device=dev)}
    ws = torch.empty(max(pa.lowrank_decode_multi_workspace_bytes(layers[0][:2]),
                         pa.lowrank_workspace_bytes(pa.PARSE_DECODE, layers[0][2], B, k)), dtype=torch.uint8, device=dev)
    pt = pa.Patterns(k, 4, subsets=subsets)
    # decode plans: built once per batch, after prefill (the subsets are fixed for every later step)
    plan_gu = pa.decode_plan(layers[0][:2], [pt, pt], pid)
    plan_dn = pa.decode_plan(layers[0][2:], [pt], pid)

    def step(s, ev=None, fused=True):
        gate, up, down = layers[s % copies]
        if ev is not None:
            ev[0].record()
        if fused:   # gate and up read the same x: one horizontally fused call (Sec. 4.4, Eq. 11-12), two launches
            pa.lowrank_decode_planned([gate, up], xs[hidden], plan_gu, [ys[inter], ys2], ws)
        else:
            pa.lowrank_decode_planned([gate], xs[hidden], plan_dn, [ys[inter]], ws)
            pa.lowrank_decode_planned([up], xs[hidden], plan_dn, [ys2], ws)
        if ev is not None:
            ev[1].record()
        pa.lowrank_decode_planned([down], xs[inter], plan_dn, [ys[hidden]], ws)
        if ev is not None:
            ev[2].record()

    ys2 = torch.empty((B, inter), dtype=torch.bfloat16, device=dev)
    steps = args.decode_steps

    def run(fused):
        for s in range(min(8, copies)):
            step(s, fused=fused)
        torch.cuda.synchronize()
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(steps):
            step(s, evs[s], fused)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        us = [sum(evs[s][i].elapsed_time(evs[s][i + 1]) for s in range(steps)) / steps * 1e3 for i in range(2)]
        return wall, us

    wall_sep, us_sep = (0.0, [0.0, 0.0]) if args.no_decode_separate else run(False)
    wall, us = run(True)
    out = {"workload": "config2: gate/up 4096->11008 (one horizontally fused call), down 11008->4096, R=2560, G=20, "
                       "k=10, B=32, 4 patterns",
           "steps": steps, "copies": copies, "distinct_groups": distinct,
           "ms_per_step": round(wall / steps * 1e3, 4), "calls": {}}
    fac = lambda n, m: distinct * gs * (n + m) * 2
    b_gu = 2 * fac(hidden, inter) + B * hidden * 2 + 2 * B * inter * 2      # x is read once for both layers
    b_dn = fac(inter, hidden) + B * (inter + hidden) * 2
    out["calls"]["gate+up"] = {"us": round(us[0], 2), "algorithmic_bytes": b_gu, "GBps": round(b_gu / us[0] / 1e3, 1)}
    out["calls"]["down"] = {"us": round(us[1], 2), "algorithmic_bytes": b_dn, "GBps": round(b_dn / us[1] / 1e3, 1)}
    out["separate_calls"] = {"gate,up_us": round(us_sep[0], 2), "down_us": round(us_sep[1], 2),
                             "ms_per_step": round(wall_sep / steps * 1e3, 4)}
    tot_bytes, tot_us = b_gu + b_dn, us[0] + us[1]
    out["eager"] = {"us_per_step": round(tot_us, 2), "GBps": round(tot_bytes / tot_us / 1e3, 1),
                    "end_to_end_GBps": round(tot_bytes * steps / wall / 1e9, 1)}
    # The same steps replayed from a HIP graph (one graph = `copies` consecutive steps = 4 * copies kernel nodes, no
    # memset nodes): what a serving loop runs.  Every replay is checked against the eager result of the same steps.
    graph_us = None
    if not args.no_decode_graph:
        for s in range(copies):
            step(s)
        torch.cuda.synchronize()
        ref = [ys[inter].clone(), ys2.clone(), ys[hidden].clone()]
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for s in range(copies):
                step(s)
        reps = max(2, steps // copies)
        same = True
        g.replay()
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        for a_, b_ in zip(ref, [ys[inter], ys2, ys[hidden]]):
            same = same and bool(torch.equal(a_.view(torch.int16), b_.view(torch.int16)))
        graph_us = e0.elapsed_time(e1) * 1e3 / (reps * copies)
        out["graph_replay"] = {"us_per_step": round(graph_us, 2), "GBps": round(tot_bytes / graph_us / 1e3, 1),
                               "steps_per_graph": copies, "replays": reps, "matches_eager_bitwise": same}
        if not same:
            graph_us = None
    best_us = graph_us if graph_us is not None else tot_us
    ach = tot_bytes / best_us / 1e3
    out["roofline"] = {"bound": "hbm",
                       "kernel": "decode_zr + decode_y over a decode plan (two calls per step: gate+up fused, down; four launches)"
                                 + (", steps replayed from a HIP graph" if graph_us is not None else ", eager launches"),
                       "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                       "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": traffic_from_profiles("decode_config2"),
                       "us_per_step": round(best_us, 2)}
    out["end_to_end_GBps"] = round(tot_bytes * steps / wall / 1e9, 1)
    return out


def bench_stack(args, torch, pa, si):
    """The full-stack workload: 32 layers x {q, k, v, o: 4096x4096; gate, up: 4096->11008; down: 11008->4096},
    factors kept at 0.6 of the dense parameter count (16 groups of 80 / 112 ranks, zero-padded to 96 / 128 for the
    operand-order layout), top-8 of 16, bf16, Gaussian factors generated on the device.  Projections are not
    chained (no attention, norm or activation here): every projection reads a fixed random input of its width.
    q/k/v and gate/up go through the horizontally fused calls.  Prefill: one prompt of 2048 tokens; decode: one
    sequence, one token per step.  Aggregated blocks are packed beforehand (timed separately)."""
    import numpy as np
    dev = "cuda"
    hidden, inter, G, k, T, NL = 4096, 11008, 16, 8, 2048, 32
    shapes = [("q", hidden, hidden), ("k", hidden, hidden), ("v", hidden, hidden), ("o", hidden, hidden),
              ("gate", hidden, inter), ("up", hidden, inter), ("down", inter, hidden)]
    rng = np.random.default_rng(si.SEED_BASE + 3)
    layers, pats, real = [], [], {}
    t_pack0 = torch.cuda.Event(enable_timing=True); t_pack1 = torch.cuda.Event(enable_timing=True)
    subs_all = []
    for l in range(NL):
        row, prow = {}, {}
        for nm, n, m in shapes:
            R, gs = si.config3_ranks(n, m, G)
            gp = (gs + 31) // 32 * 32
            real[nm] = (gs, gp)
            Vt = (torch.randn((G * gp, n), device=dev) * 0.02).to(torch.bfloat16)
            Ut = (torch.randn((G * gp, m), device=dev) * 0.02).to(torch.bfloat16)
            row[nm] = pa.Layer(Vt, Ut, n, m, G * gp, G, pa.PARSE_MFMA16)
            sub = torch.from_numpy(np.sort(rng.choice(G, size=k, replace=False)).astype(np.int32)[None, :]).to(dev)
            subs_all.append((l, nm, sub))
            prow[nm] = sub
        layers.append(row); pats.append(prow)
    torch.cuda.synchronize()
    t_pack0.record()
    for l in range(NL):
        for nm, n, m in shapes:
            Vs, Us = pa.pack_patterns(layers[l][nm], pats[l][nm], k, k, None, None, 1)
            pats[l][nm] = pa.Patterns(k, 1, Vs, Us, subsets=pats[l][nm])
    t_pack1.record(); torch.cuda.synchronize()
    pack_ms = t_pack0.elapsed_time(t_pack1)
    Xh = torch.randn((T, hidden), device=dev).to(torch.bfloat16); Xi = torch.randn((T, inter), device=dev).to(torch.bfloat16)
    off = torch.tensor([0, T], dtype=torch.int32, device=dev); pid = torch.zeros(1, dtype=torch.int32, device=dev)
    Yh = [torch.empty((T, hidden), dtype=torch.bfloat16, device=dev) for _ in range(3)]
    Yi = [torch.empty((T, inter), dtype=torch.bfloat16, device=dev) for _ in range(2)]
    L0 = layers[0]
    P0 = pats[0]
    ws_qkv = torch.empty(max(pa.lowrank_prefill_multi_workspace_bytes([L0["q"], L0["k"], L0["v"]], [P0["q"], P0["k"], P0["v"]], T),
                             int(pa.lowrank_workspace_bytes(pa.PARSE_PREFILL, L0["o"], T, k, 1, 1))), dtype=torch.uint8, device=dev)
    ws_gu = torch.empty(max(pa.lowrank_prefill_multi_workspace_bytes([L0["gate"], L0["up"]], [P0["gate"], P0["up"]], T),
                            int(pa.lowrank_workspace_bytes(pa.PARSE_PREFILL, L0["down"], T, k, 1, 1))), dtype=torch.uint8, device=dev)
    wsd = torch.empty(max(pa.lowrank_decode_multi_workspace_bytes([L0["q"], L0["k"], L0["v"]]),
                          pa.lowrank_decode_multi_workspace_bytes([L0["gate"], L0["up"]]),
                          pa.lowrank_workspace_bytes(pa.PARSE_DECODE, L0["o"], 1, k),
                          pa.lowrank_workspace_bytes(pa.PARSE_DECODE, L0["down"], 1, k)), dtype=torch.uint8, device=dev)

    def prefill():
        for l in range(NL):
            Ly, Pt = layers[l], pats[l]
            pa.lowrank_prefill_multi([Ly["q"], Ly["k"], Ly["v"]], [Pt["q"], Pt["k"], Pt["v"]], Xh, off, pid, Yh, ws_qkv)
            pa.lowrank_forward(pa.PARSE_PREFILL, Ly["o"], Pt["o"], Xh, off, pid, Yh[0], ws_qkv)
            pa.lowrank_prefill_multi([Ly["gate"], Ly["up"]], [Pt["gate"], Pt["up"]], Xh, off, pid, Yi, ws_gu)
            pa.lowrank_forward(pa.PARSE_PREFILL, Ly["down"], Pt["down"], Xi, off, pid, Yh[0], ws_gu)

    xh1, xi1 = Xh[:1].contiguous(), Xi[:1].contiguous()
    yh1 = [torch.empty((1, hidden), dtype=torch.bfloat16, device=dev) for _ in range(3)]
    yi1 = [torch.empty((1, inter), dtype=torch.bfloat16, device=dev) for _ in range(2)]

    # decode plans, once per batch (the subsets are fixed after prefill): one per horizontally fused call of every layer
    dplans = []
    for l in range(NL):
        Ly, Pt = layers[l], pats[l]
        dplans.append({"qkv": pa.decode_plan([Ly["q"], Ly["k"], Ly["v"]], [Pt["q"], Pt["k"], Pt["v"]], pid),
                       "o": pa.decode_plan([Ly["o"]], [Pt["o"]], pid),
                       "gu": pa.decode_plan([Ly["gate"], Ly["up"]], [Pt["gate"], Pt["up"]], pid),
                       "down": pa.decode_plan([Ly["down"]], [Pt["down"]], pid)})

    def decode_step():
        for l in range(NL):
            Ly, D = layers[l], dplans[l]
            pa.lowrank_decode_planned([Ly["q"], Ly["k"], Ly["v"]], xh1, D["qkv"], yh1, wsd)
            pa.lowrank_decode_planned([Ly["o"]], xh1, D["o"], yh1[:1], wsd)
            pa.lowrank_decode_planned([Ly["gate"], Ly["up"]], xh1, D["gu"], yi1, wsd)
            pa.lowrank_decode_planned([Ly["down"]], xi1, D["down"], yh1[:1], wsd)

    def wall(fn, reps):
        fn(); torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps

    t_pre = wall(prefill, 3)
    t_dec = wall(decode_step, args.stack_decode_steps)
    # the same decode step captured once as a HIP graph and replayed (384 kernel nodes, no other node kinds)
    t_graph = None
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            decode_step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            decode_step()
        ref = [y.clone() for y in yh1 + yi1]
        t_graph = wall(graph.replay, args.stack_decode_steps)
        same = all(torch.equal(a, b) for a, b in zip(ref, yh1 + yi1))     # replays write the same bits as eager
        assert same, "graph replay differs from the eager step"
    except Exception as exc:   # capture is an optimisation of the launch path, not part of the method
        t_graph = f"unavailable: {type(exc).__name__}"
    flops = sum(2.0 * T * k * real[nm][0] * (n + m) for nm, n, m in shapes) * NL        # real (unpadded) ranks
    dbytes = sum(k * real[nm][0] * (n + m) * 2 + (n + m) * 2 for nm, n, m in shapes) * NL
    stored = sum(G * real[nm][1] * (n + m) * 2 for nm, n, m in shapes) * NL
    return {"workload": "32 layers x 7 projections, kept ratio 0.6 (16 groups of 80/112 ranks, padded to 96/128), top-8; "
                        "prefill 1 x 2048 tokens, decode 1 sequence",
            "stored_factor_GB": round(stored / 1e9, 2), "aggregation_ms_all_224_patterns": round(pack_ms, 2),
            "prefill_ms": round(t_pre * 1e3, 3), "prefill_TFLOPs": round(flops / t_pre / 1e12, 1),
            "prefill_frac_of_mfma_peak": round(flops / t_pre / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
            "decode_frac_of_hbm_peak": round(dbytes / t_dec / 1e9 / HBM_PEAK_GBS, 4),
            "prefill_tokens_per_s": round(T / t_pre, 1),
            "decode_ms_per_step": round(t_dec * 1e3, 3), "decode_GBps": round(dbytes / t_dec / 1e9, 1),
            "decode_ms_per_step_graph": round(t_graph * 1e3, 3) if isinstance(t_graph, float) else t_graph,
            "decode_GBps_graph": round(dbytes / t_graph / 1e9, 1) if isinstance(t_graph, float) else None,
            "launches_per_decode_step": NL * 4 * 2,
            "cpu_baseline": stack_cpu_baseline(layers[0], pats[0], real, shapes, T, k, G, Xh, Xi, flops, dbytes)}


def stack_cpu_baseline(L0, P0, real, shapes, T, k, G, Xh, Xi, flops_total, dbytes_total):
    """The oracle on a sample of the full-stack workload: layer 0's seven projections, prefill rows 0..127 and two decode
    steps of one sequence (dense reconstruction and apply in float64), extrapolated by flop / byte count."""
    import numpy as np
    from oracle import parse_oracle as po
    pre_flops = dec_bytes = t_pre = t_dec = 0.0
    for nm, n, m in shapes:
        lay = L0[nm]
        # stored (operand-order) factors back to row-major through the documented index map
        R = lay.R
        Vt = lay.Vt.view(R // 32, n // 16, 2, 32, 8).permute(0, 3, 1, 2, 4).reshape(R, n).float().cpu().numpy().astype(np.float64)
        Ut = lay.Ut.view(R // 16, m // 32, 2, 32, 8).permute(0, 2, 4, 1, 3).reshape(R, m).float().cpu().numpy().astype(np.float64)
        gp = R // G
        sub = P0[nm].subsets.cpu().numpy()
        X = (Xh if n == Xh.shape[1] else Xi)[:128].float().cpu().numpy().astype(np.float64)
        t0 = time.perf_counter()
        po.forward(Ut.T, np.ones(R), Vt, gp, X, [0, 128], sub)
        t_pre += time.perf_counter() - t0
        pre_flops += 2.0 * 128 * k * real[nm][0] * (n + m)
        t0 = time.perf_counter()
        for _ in range(2):
            po.decode_step(Ut.T, np.ones(R), Vt, gp, X[:1], sub)
            dec_bytes += k * real[nm][0] * (n + m) * 2
        t_dec += time.perf_counter() - t0
    return {"kind": "oracle", "cores": len(os.sched_getaffinity(0)), "seconds": round(t_pre + t_dec, 2),
            "sample": "layer 0's seven projections: prefill rows 0..127 and two decode steps of one sequence",
            "prefill_TFLOPs_sample": round(pre_flops / t_pre / 1e12, 5),
            "extrapolated_prefill_s": round(t_pre * flops_total / pre_flops, 1),
            "decode_GBps_sample": round(dec_bytes / t_dec / 1e9, 3),
            "extrapolated_decode_s_per_step": round(t_dec * dbytes_total / dec_bytes, 1),
            "note": "extrapolated linearly by flop / byte count; the dense reconstruction of W_S dominates both samples"}


def bench_peaks(torch, pa):
    """Achievable peaks on this machine, measured with the library's probe kernels (HIP events around 5 launches, best
    of 3): the bf16 matrix-instruction loop on constant and on random operands, and read-only / copy streams at the
    sizes the workloads move (a decode call's factors, a decode step, a large stream)."""
    dev = "cuda"
    out = {}
    def timed(fn, reps=5):
        best = 1e30
        for _ in range(3):
            fn(); torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                fn()
            e1.record(); torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1) / reps)
        return best * 1e-3
    wgs, iters = 1024, 2048
    sink = torch.empty(wgs * 256, dtype=torch.float32, device=dev)
    flop = wgs * 4 * iters * 8 * 32768.0
    for nm, data in (("constant_operands", torch.full((24 * 1024 // 2,), 1.0, dtype=torch.bfloat16, device=dev)),
                     ("random_operands", torch.randn(24 * 1024 // 2, device=dev).to(torch.bfloat16))):
        t = timed(lambda: pa.probe_mfma_bf16(data, wgs, iters, sink))
        out["mfma_bf16_TFLOPs_" + nm] = round(flop / t / 1e12, 1)
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev); src.random_(0, 255)
    dst = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
    s32 = torch.zeros(1, dtype=torch.int32, device=dev)
    reads = {}
    for mb in (16, 64, 128, 224, 1024):
        nbytes = mb << 20
        for nwg in (128, 256):
            if nbytes % (nwg * 65536):
                continue
            t = timed(lambda: pa.probe_read(src, nbytes, nwg, s32))
            reads[f"{mb}MiB_{nwg}wg"] = round(nbytes / t / 1e9, 1)
    out["read_stream_GBps"] = reads
    out["copy_GBps"] = {f"{mb}MiB": round(2.0 * (mb << 20) / timed(lambda: pa.probe_copy(src, dst, mb << 20)) / 1e9, 1)
                        for mb in (64, 256)}
    # The vendor's GEMM (hipBLASLt behind torch.matmul) on the two products of the prefill workloads with ONE shared
    # factor pair for all rows -- no per-prompt patterns, so it reads 117 MB less than the routed call at 8 x 512 -- as
    # a yardstick for what these shapes reach on this machine.  Measurement context only: nothing in the path uses it.
    del src, dst
    torch.cuda.empty_cache()
    n = m = 4096; rS = 1024
    Vd = (torch.randn((n, rS), device=dev) * 0.02).to(torch.bfloat16)
    Ud = (torch.randn((rS, m), device=dev) * 0.02).to(torch.bfloat16)
    vend = {}
    for T in (4096, 32768):
        Xd = torch.randn((T, n), device=dev).to(torch.bfloat16)
        Zd = torch.empty((T, rS), dtype=torch.bfloat16, device=dev); Yd = torch.empty((T, m), dtype=torch.bfloat16, device=dev)
        def pair():
            torch.matmul(Xd, Vd, out=Zd); torch.matmul(Zd, Ud, out=Yd)
        t = timed(pair, reps=10)
        vend[f"{T}_rows"] = {"us": round(t * 1e6, 1), "TFLOPs": round(2.0 * T * rS * (n + m) / t / 1e12, 1)}
        del Xd, Zd, Yd
    out["vendor_gemm_pair_one_shared_factor"] = vend
    out["note"] = ("read streams smaller than the 256 MiB last-level cache are re-read from it on the repeated launches; "
                   "the 1 GiB stream comes from HBM.  copy counts bytes read plus bytes written.  vendor_gemm_pair: "
                   "torch.matmul (hipBLASLt) X[T,4096] @ V[4096,1024] then Z @ U[1024,4096], bf16, back to back.")
    return out


def bench_stress(args, torch, pa, si):
    """Pattern-cache and grouped-execution stress: 256 prompts whose embeddings come from 16 Gaussian clusters (4096-d,
    spread 0.1), lengths uniform in 32..2048 tokens, MLP-shaped layers (gate, up: 4096->11008, down: 11008->4096, R=2560
    in 20 groups, top-10), cosine threshold 0.9.  One pass = cache probe with route-on-miss for the three routed matrices
    -> bucket -> aggregation of the new cache entries (per layer) -> prefill plan (rows grouped by pattern) -> planned
    prefill of gate, up and down, all prompts of a pattern in the same tiles.  Factors are Gaussian bf16 generated on the
    device (timing; parity at this size is covered by the tests); tokens are N(0,1)."""
    import numpy as np
    from oracle import parse_oracle as po
    dev = "cuda"
    E, cid, off_h, Wr_h = si.config4_embeddings()
    P, d, G, k, R, hidden, inter, L = E.shape[0], E.shape[1], 20, 10, 2560, 4096, 11008, 3
    gs, rS = R // G, k * (R // G)
    rows = int(off_h[-1])
    shapes = [("gate", hidden, inter), ("up", hidden, inter), ("down", inter, hidden)]
    n_slots = 32
    layers_rm, layers = [], []
    for nm, n, m in shapes:
        Vt = (torch.randn((R, n), device=dev) * 0.02).to(torch.bfloat16)
        Ut = (torch.randn((R, m), device=dev) * 0.02).to(torch.bfloat16)
        rm = pa.Layer(Vt, Ut, n, m, R, G, pa.PARSE_ROWMAJOR)
        layers_rm.append(rm); layers.append(pa.layer_to_mfma16(rm))
    Xh = torch.randn((rows, hidden), device=dev).to(torch.bfloat16)
    Xi = torch.randn((rows, inter), device=dev).to(torch.bfloat16)
    Ys = [torch.empty((rows, m), dtype=torch.bfloat16, device=dev) for _, _, m in shapes]
    Ed, off, Wr = torch.from_numpy(E).to(dev), torch.from_numpy(off_h).to(dev), torch.from_numpy(Wr_h).to(dev)
    cache = pa.Cache(n_slots, d, L, k, P)
    entry = torch.empty(P, dtype=torch.int32, device=dev); hit = torch.empty(P, dtype=torch.uint8, device=dev)
    sim = torch.empty(P, dtype=torch.float32, device=dev); subs = torch.empty((P, L, k), dtype=torch.int32, device=dev)
    bucket_out = (torch.empty(P, dtype=torch.int32, device=dev), torch.empty(P, dtype=torch.int32, device=dev),
                  torch.empty(P + 1, dtype=torch.int32, device=dev), torch.empty(1, dtype=torch.int32, device=dev),
                  torch.empty(P, dtype=torch.int32, device=dev))
    packed = [(torch.empty((n_slots, rS, n), dtype=torch.bfloat16, device=dev),
               torch.empty((n_slots, rS, m), dtype=torch.bfloat16, device=dev)) for _, n, m in shapes]
    pts = [pa.Patterns(k, n_slots, Vs, Us) for Vs, Us in packed]
    plan = torch.empty(pa.prefill_plan_bytes(rows, P, n_slots), dtype=torch.uint8, device=dev)
    ws = torch.empty(max(pa.lowrank_prefill_planned_workspace_bytes(l, rows, P, k, n_slots) for l in layers),
                     dtype=torch.uint8, device=dev)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(6)]

    def one_pass():
        ev[0].record()
        cache.lookup_or_route(Ed, 0.9, Wr, entry, hit, sim, subs)
        pa.bucket_patterns(subs.view(P, L * k), L * k, L * k, bucket_out)
        ev[1].record()
        for l in range(L):   # aggregation once per new cache entry and layer (slot = cache entry)
            pa.pack_new_entries(layers[l], subs.view(P, L * k)[:, l * k:], L * k, k, entry, hit, packed[l][0], packed[l][1])
        ev[2].record()
        pa.prefill_plan(off, entry, rows, n_slots, plan)
        ev[3].record()
        pa.lowrank_prefill_planned(layers[0], pts[0], Xh, off, entry, plan, Ys[0], ws)   # gate and up read the same rows
        pa.lowrank_prefill_planned(layers[1], pts[1], Xh, off, entry, plan, Ys[1], ws)
        ev[4].record()
        pa.lowrank_prefill_planned(layers[2], pts[2], Xi, off, entry, plan, Ys[2], ws)
        ev[5].record()
        torch.cuda.synchronize()
        return [ev[i].elapsed_time(ev[i + 1]) for i in range(5)]

    cold = one_pass()                                      # empty cache: one miss per cluster, 16 x 3 aggregations
    hits_cold, entries = int(hit.sum().item()), cache.count()
    assert torch.equal(subs.cpu(), torch.from_numpy(po.PatternCache(n_slots, d, L, k).lookup_or_route(E, 0.9, Wr_h)[2]))
    warm = [one_pass() for _ in range(3)][-1]              # every prompt hits: nothing is routed or aggregated
    hits_warm = int(hit.sum().item())
    words = plan.view(torch.int32)[:4].cpu().numpy()
    vrows = int(words[1])
    flops = sum(2.0 * rows * rS * (n + m) for _, n, m in shapes)
    fwd_ms = warm[3] + warm[4]
    # the oracle on 4 prompts per layer (dense reconstruction and apply in float64), extrapolated by flop count
    t0 = time.perf_counter(); done_flops = 0.0
    sub_h = subs.cpu().numpy()
    for l, (nm, n, m) in enumerate(shapes):
        Vt = layers_rm[l].Vt.float().cpu().numpy().astype(np.float64); Ut = layers_rm[l].Ut.float().cpu().numpy().astype(np.float64)
        Xsrc = Xh if n == hidden else Xi
        for p in (0, 1, 2, 3):
            a, b = int(off_h[p]), int(off_h[p + 1])
            po.forward(Ut.T, np.ones(R), Vt, gs, Xsrc[a:b].float().cpu().numpy().astype(np.float64), [0, b - a], sub_h[p:p + 1, l])
            done_flops += 2.0 * (b - a) * rS * (n + m)
    dt = time.perf_counter() - t0
    cache.close()
    return {"workload": "config4: 256 prompts, 16 clusters (spread 0.1), lengths U{32..2048}, gate/up 4096->11008 and down "
                        "11008->4096, R=2560 in 20 groups, top-10, tau=0.9; one pass = probe, bucket, aggregation, plan, "
                        "planned prefill of the three layers",
            "prompts": P, "tokens": rows, "cache_entries": entries, "hits_first_pass": hits_cold,
            "hit_rate_first_pass": round(hits_cold / P, 4), "expected_hit_rate": round((P - 16) / P, 4),
            "hits_warm_pass": hits_warm, "patterns": int(bucket_out[3].item()),
            "launches_per_layer_forward": 2, "tokens_per_launch": rows,
            "virtual_rows": vrows, "tile_padding_overhead": round(vrows / rows - 1.0, 4),
            "first_pass_ms": {"probe+bucket": round(cold[0], 3), "aggregate_16x3": round(cold[1], 3), "plan": round(cold[2], 3),
                              "gate+up": round(cold[3], 3), "down": round(cold[4], 3)},
            "warm_pass_ms": {"probe+bucket": round(warm[0], 3), "aggregate": round(warm[1], 3), "plan": round(warm[2], 3),
                             "gate+up": round(warm[3], 3), "down": round(warm[4], 3)},
            "forward_TFLOPs": round(flops / (fwd_ms * 1e-3) / 1e12, 1),
            "forward_frac_of_mfma_peak": round(flops / (fwd_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
            "pass_TFLOPs": round(flops / (sum(warm) * 1e-3) / 1e12, 1),
            "cpu_baseline": {"value": round(done_flops / dt / 1e12, 5), "unit": "TFLOP/s", "cores": len(os.sched_getaffinity(0)),
                             "kind": "oracle", "sample": f"4 prompts per layer, {dt:.1f} s; extrapolated to the whole pass: "
                                                         f"{flops / (done_flops / dt):.0f} s"}}


def cpu_baseline(w, flops):
    """The CPU oracle as it stands, timed on the host cores on the same workload (bounded sample)."""
    import numpy as np
    from oracle import parse_oracle as po
    from helpers import oracle_factors
    lay = w.layers[0]
    cores = len(os.sched_getaffinity(0))
    Xv = w.X_values()
    U0, sg, V = oracle_factors(lay)
    # sample: whole prompts of the workload, pass after pass, for roughly 10 s (at least one prompt)
    done, t0 = 0, time.perf_counter()
    budget = 10.0
    while True:
        p = done % w.P
        off = w.tok_offsets[p:p + 2] - w.tok_offsets[p]
        a, b = int(w.tok_offsets[p]), int(w.tok_offsets[p + 1])
        E = po.pool(Xv[a:b], off)
        subs, _ = po.route(E, w.Wr[0], w.k)
        po.pack(lay.Vt_store, lay.Ut_store, subs[0], lay.gs)
        po.forward(U0, sg, V, lay.gs, Xv[a:b], off, subs)
        done += 1
        if time.perf_counter() - t0 > budget:
            break
    dt = time.perf_counter() - t0
    frac = done / w.P
    return {"value": round(flops * frac / dt / 1e12, 5), "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": f"{done} prompts ({frac:.1f} passes over the {w.P} prompts of the same workload: pool, route, pack, "
                      f"dense reconstruction and apply in float64), {dt:.1f} s", "seconds": round(dt, 2)}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (the layer shards by prompts/"
              "sequences with no exchange step); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2605_08568_amd as pa
    import synth_inputs as si
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    dec = None
    if args.only_decode:
        print(json.dumps({"decode": bench_decode(args, torch, pa, si)}))
        return
    if args.only_stress:
        print(json.dumps({"stress": bench_stress(args, torch, pa, si)}))
        return
    if args.only_peaks:
        print(json.dumps({"achievable": bench_peaks(torch, pa)}))
        return
    pre = bench_prefill(args, torch, pa, si)
    w = pre.pop("workload")
    scaled = None
    if not args.no_token_scaled and args.tokens == 512 and not args.no_extras:
        # side record: the same step on prompts of 4096 tokens (8 x 4096 rows, large tiles in both products); the forward
        # figure is the one timed inside the full steps (HIP events around the call), not a back-to-back loop
        a2 = argparse.Namespace(**{**vars(args), "tokens": 4096, "steps": 10, "warmup": 2, "no_extras": True,
                                   "no_prefill_graph": True})
        p2 = bench_prefill(a2, torch, pa, si)
        p2.pop("workload")
        scaled = {"workload": f"{args.prompts} prompts x 4096 tokens, otherwise as config1", "steps": 10,
                  "ms_per_step_eager": round(p2["ms_per_step"], 4), "step_TFLOPs": round(p2["value"], 1),
                  "rows_us": p2["rows_us"], "forward_in_step_us": p2["roofline"]["launch_us"],
                  "forward_TFLOPs": p2["roofline"]["achieved"], "forward_frac_of_mfma_peak": p2["roofline"]["frac"],
                  "kernel": "gemm_lds<256,256,2x2,BK32,S4> + gemm_lds<256,256,2x4,BK32,S4> (one planned forward call)"}
        del p2
        torch.cuda.empty_cache()
    if not args.no_decode:
        dec = bench_decode(args, torch, pa, si)
    stack = bench_stack(args, torch, pa, si) if args.stack else None
    base = None if args.no_cpu_baseline else cpu_baseline(w, pre["flops_per_step"])
    lay = w.layers[0]
    line = {
        "metric": "routed low-rank linear: prefill TFLOP/s (%MFMA peak); decode GB/s (%HBM peak)",
        "value": round(pre["value"], 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(pre["ms_per_step"], 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"config1: q_proj-shaped prefill, bf16, {lay.m}x{lay.n}, R={lay.R} in {lay.G} groups of "
                               f"{lay.gs}, top-{w.k}, {w.P} prompts x {args.tokens} tokens, one routed subset per prompt",
                   "step": "pool, cache probe (route-on-miss), buckets + plan (one launch), pack of new cache entries, forward; "
                           "warm cache in the timed steps, cold_step_ms = the same step with an empty cache",
                   "launch_mode": pre["launch_mode"] + (f": the K timed steps are replays of a HIP graph of "
                                                        f"{(pre['graph_replay'] or {}).get('steps_per_graph', 2)} "
                                                        "consecutive steps, checked bitwise against the eager steps; "
                                                        "rows_us and roofline come from the eager steps"
                                                        if pre["launch_mode"] == "graph" else "")},
        "roofline": pre["roofline"],
        "cpu_baseline": base,
        "rows_us": pre["rows_us"],
        "eager_ms_per_step": round(pre["eager_ms_per_step"], 4),
        "graph_replay": pre["graph_replay"],
        "cache_hits_last_step": pre["cache_hits"],
        "forward_us_by_schedule": pre["forward_us_by_schedule"],
        "cold_step_ms": pre["cold_step_ms"],
        "rank_granular_us": pre["rank_granular_us"],
        "two_batches_in_flight": pre["two_batches_in_flight"],
        "token_scaled_8x4096": scaled,
        "decode": dec,
    }
    if not args.no_peaks:
        line["achievable"] = bench_peaks(torch, pa)
    if stack is not None:
        line["stack"] = stack
    if args.stress:
        line["stress"] = bench_stress(args, torch, pa, si)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
