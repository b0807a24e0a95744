#!/usr/bin/env python3
"""Benchmark of the locality-constrained block-sparse attention hot path on one MI355X.

One STEP = one chunk of latent frames through every layer of the workload: per layer
lcsa_kv_cache_append -> lcsa_pool_select_blocks -> lcsa_sparse_attn_fwd, each layer with its own seeded
Q/K/V and its own sliding-window cache (already primed, so the timed step runs in steady state: append
evicts the oldest frames, attention sees a full window).  Inputs are resident in HBM before the timed
region.  Prints ONE JSON line: the headline workload (default: paper-scale, the configuration the metric is
quoted on), then, outside the timed region, short measurements of the other benchmark configurations
("other_workloads"), what the chip sustains on trivial loops ("measured_peaks"), per-workgroup time stamps of
the attention kernel ("attn_timers") and the CPU oracle on a bounded sample ("cpu_baseline").

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload paper|small|ultra|4k|tiny]
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import re
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 / fp16 matrix peak
PEAK_F32_TFLOPS = 157.3        # vector fp32 (the generic kernels of the Tiny configuration)
PEAK_HBM_GBS = 8000.0

WORKLOAD_TEXT = {
    "tiny": "tiny: 6x8 tokens/frame, 1 head, d=32, fp32, 2 query + 2 cached frames, 4x4 tiles, radius 4, top-k 4",
    "paper": "paper-scale 768x1408: 48x88 tokens/frame, 2 query + 4 cached frames, 8x16 tiles, radius 24, top-k 32, 30 layer calls",
    "small": "small-video 384x704: 24x44 tokens/frame, 2 query + 4 cached frames, 8x16 tiles, radius 16, top-k 16",
    "ultra": "ultra-high-res 1440x2560: 90x160 tokens/frame, 2 query + 4 cached frames, 8x16 tiles, radius 24, top-k 32",
    "4k": "4k streaming 2160x3840: 135x240 tokens/frame, 1 query frame, ring of 6 frames, 8x16 tiles, radius 24, top-k 32",
}


def attn_traffic_from_profiles(workload: str, topk: int):
    """HBM-side bytes of one attention launch (L2 <-> fabric) as the rocprofv3 --pmc summaries under profiles/
    state them: a line `TRAFFIC attn_mfma_kernel workload=<w> topk=<k> fetch_bytes=<f> write_bytes=<w>`
    (FETCH_SIZE and WRITE_SIZE already scaled by the factors a plain copy of known size gives, as that file
    says).  Counters cannot be read from inside this script; None if no summary covers the workload."""
    pat = re.compile(rf"^TRAFFIC attn_mfma_kernel workload={workload} topk={topk} fetch_bytes=([0-9.e+]+) write_bytes=([0-9.e+]+)")
    pdir = os.path.join(ROOT, "profiles")
    if not os.path.isdir(pdir):
        return None
    for name in sorted(os.listdir(pdir)):
        if not name.endswith(".txt"):
            continue
        for line in open(os.path.join(pdir, name)):
            m = pat.match(line)
            if m:
                return float(m.group(1)) + float(m.group(2))
    return None


class Aids:
    """libbench_probe.so: measurement aids that are not part of the library (built by __graft_entry__.build())."""

    def __init__(self):
        path = os.path.join(ROOT, "libbench_probe.so")
        self.lib = ctypes.CDLL(path) if os.path.exists(path) else None
        if self.lib:
            vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
            self.lib.bench_probe_mfma_bf16.argtypes = [vp, i32, i32, vp]
            self.lib.bench_mock_loop.argtypes = [i32, vp, vp, i32, i32, vp]
            self.lib.bench_attn_timed.argtypes = [vp, vp, i64, i64, vp, vp, vp, vp, i64, i64, f32, vp, vp]
            for f in (self.lib.bench_probe_mfma_bf16, self.lib.bench_mock_loop, self.lib.bench_attn_timed):
                f.restype = i32


def valid_tokens_per_block(w, tile_t):
    ty, tx = -(-w.grid_h // w.tile_h), -(-w.grid_w // w.tile_w)
    vh = np.minimum(w.tile_h, w.grid_h - np.arange(ty) * w.tile_h)
    vw = np.minimum(w.tile_w, w.grid_w - np.arange(tx) * w.tile_w)
    return (vh[:, None] * vw[None, :]).reshape(-1) * tile_t


def attention_flop(sel_idx, valid_tok, n_qb, nb, d):
    """(useful, issued) flop of one attention launch from the selection actually made: 4 d sum valid_q valid_k;
    issued = the same with valid counts rounded up to the 32 x 32 tiles the matrix-core kernel computes."""
    idx = sel_idx.cpu().numpy()
    up32 = -(-valid_tok // 32) * 32
    q_tiles = np.arange(n_qb) % nb
    kvalid = np.where(idx >= 0, valid_tok[np.maximum(idx, 0) % nb], 0).sum(axis=-1)   # [h][qb]
    kiss = np.where(idx >= 0, up32[np.maximum(idx, 0) % nb], 0).sum(axis=-1)
    return (4.0 * d * float((valid_tok[q_tiles][None, :] * kvalid).sum()),
            4.0 * d * float((up32[q_tiles][None, :] * kiss).sum()))


def measure(torch, B, wl, args, name, steps, warmup, n_layers=None):
    """Sets up the layer calls of a workload (caches primed), times `steps` steps and returns the figures plus
    the live objects (for the aids that run afterwards)."""
    w = wl.WORKLOADS[name]
    n_layers = n_layers or args.layers or w.n_layers
    topk = args.topk or w.topk
    radius = w.radius if args.radius is None else args.radius
    tile_t = 1
    if args.blocks:
        tile_t, th, tw = (int(x) for x in args.blocks.split(","))
        w = wl.with_overrides(w, tile_h=th, tile_w=tw)
    if args.grid:
        gh, gw = (int(x) for x in args.grid.split(","))
        w = wl.with_overrides(w, grid_h=gh, grid_w=gw)
    if args.cache_frames:
        w = wl.with_overrides(w, cache_frames=args.cache_frames)
    bf16 = w.dtype == "bf16"
    g = B.Geom(w.heads, w.head_dim, w.grid_h, w.grid_w, w.tile_h, w.tile_w, w.q_frames, w.cache_frames,
               radius, radius, topk, dtype=B.LCSA_BF16 if bf16 else B.LCSA_F32, tile_t=tile_t)
    n_qb = g.n_qb
    policy = {"sliding": B.LCSA_EVICT_SLIDING, "headwise": B.LCSA_EVICT_IMPORTANCE_HEADWISE,
              "uniform": B.LCSA_EVICT_IMPORTANCE_UNIFORM}[args.eviction]
    scoring = policy != B.LCSA_EVICT_SLIDING

    def dev(x):
        if bf16:
            return torch.from_numpy(wl.bf16_bits(x).view(np.int16)).view(torch.bfloat16).cuda()
        return torch.from_numpy(np.ascontiguousarray(x, np.float32)).cuda()

    # ---- setup: seeded inputs per layer (host, threads), caches primed ---------------------------
    t0 = time.time()

    def gen(layer):
        s = wl.ChunkStream(w, layer)
        return [s.next() for _ in range(w.prime_chunks + 1)]

    layers = []
    host_layer0 = None
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
        for layer, chunks in enumerate(pool.map(gen, range(n_layers))):
            cache = B.lcsa_cache_init(g)
            if policy != B.LCSA_EVICT_SLIDING:
                B.lcsa_cache_set_eviction(cache, policy)
            dchunks = [tuple(dev(x) for x in c) for c in chunks]
            # fill the ring with all chunks of the stream; a timed step then re-appends them in turn,
            # so the window always holds the same frames (a static scene) and every append evicts
            for (qd, kd, vd) in dchunks:
                B.lcsa_kv_cache_append(cache, kd, vd, w.q_frames)
            layers.append(dict(
                cache=cache, chunks=dchunks, turn=0,
                pq=torch.empty(g.heads, n_qb, g.head_dim, dtype=torch.float32, device="cuda"),
                sel_idx=torch.empty(g.heads, n_qb, topk, dtype=torch.int32, device="cuda"),
                sel_cnt=torch.empty(g.heads, n_qb, dtype=torch.int32, device="cuda"),
                o=torch.empty_like(dchunks[0][0])))
            if layer == 0:
                host_layer0 = chunks
    torch.cuda.synchronize()
    setup_s = time.time() - t0

    def layer_call(L, ev=None, attn_ev=None):
        q, k, v = L["chunks"][L["turn"] % len(L["chunks"])]
        L["turn"] += 1
        B.lcsa_kv_cache_append(L["cache"], k, v, w.q_frames)
        if ev: ev[0].record()
        if args.two_calls:
            B.lcsa_pool_blocks(g, q, w.q_frames, L["pq"])
            if ev: ev[1].record()
            B.lcsa_select_blocks(g, L["pq"], L["cache"], L["sel_idx"], L["sel_cnt"], want_gap=False)
        else:
            if ev: ev[1].record()
            B.lcsa_pool_select_blocks(g, q, L["cache"], L["pq"], L["sel_idx"], L["sel_cnt"], want_gap=False)
        if ev: ev[2].record()
        if attn_ev: attn_ev[0].record()
        B.lcsa_sparse_attn_fwd(g, q, L["cache"], L["sel_idx"], L["sel_cnt"], L["o"])
        if attn_ev: attn_ev[1].record()
        if ev: ev[3].record()
        if scoring:
            B.lcsa_block_importance(g, L["pq"], L["cache"])     # scores the visible groups for the next append
        if ev: ev[5].record()

    for _ in range(warmup):
        for L in layers:
            layer_call(L)
    torch.cuda.synchronize()

    # ---- timed region: exactly `steps` steps; HIP events around every attention launch ------------
    # (all launches go to torch's current stream, which is the stream these events are recorded on)
    attn_ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in layers]
               for _ in range(steps)]
    graphs = []
    if args.graph:
        # one graph per position of the chunk rotation: the inputs of a captured call are fixed
        for _ in range(len(layers[0]["chunks"])):
            gph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gph):
                for L in layers:
                    layer_call(L)
            graphs.append(gph)
        for s_ in range(warmup):
            graphs[s_ % len(graphs)].replay()
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for s in range(steps):
        if args.graph:
            graphs[(warmup + s) % len(graphs)].replay()
        else:
            for L, (e0, e1) in zip(layers, attn_ev[s]):
                layer_call(L, attn_ev=(e0, e1))
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    ms_per_step = elapsed * 1e3 / steps
    ms_per_layer = ms_per_step / n_layers
    attn_ms = None if args.graph else np.array([[e0.elapsed_time(e1) for (e0, e1) in step] for step in attn_ev])

    # ---- untimed breakdown pass: events between the calls ------------------------------------------
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in layers]
    for L, e in zip(layers, ev):
        e[4].record()
        layer_call(L, e)
    torch.cuda.synchronize()
    brk = np.array([[e[4].elapsed_time(e[0]), e[0].elapsed_time(e[1]), e[1].elapsed_time(e[2]), e[2].elapsed_time(e[3]),
                     e[3].elapsed_time(e[5])] for e in ev]).mean(axis=0)
    if attn_ms is None:      # launches inside a graph carry no events: the attention launches of this eager pass stand in
        attn_ms = np.array([[e[2].elapsed_time(e[3]) for e in ev]])

    # ---- the same step replayed from captured HIP graphs, beside the eager figure (untimed region of its own) ----
    replay_ms_per_layer = None
    if args.graph_too and not args.graph:
        gs = []
        for _ in range(len(layers[0]["chunks"])):
            gph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gph):
                for L in layers:
                    layer_call(L)
            gs.append(gph)
        for s_ in range(max(warmup, 1)):
            gs[s_ % len(gs)].replay()
        torch.cuda.synchronize()
        t_g = time.perf_counter()
        for s_ in range(steps):
            gs[(warmup + s_) % len(gs)].replay()
        torch.cuda.synchronize()
        replay_ms_per_layer = (time.perf_counter() - t_g) * 1e3 / steps / n_layers
        del gs

    # ---- algorithmic work of one attention launch (from the selection actually made) ---------------
    valid_tok = valid_tokens_per_block(w, tile_t)
    flops = [attention_flop(L["sel_idx"], valid_tok, n_qb, g.nb, g.head_dim) for L in layers]
    useful_flop, issued_flop = float(np.mean([f[0] for f in flops])), float(np.mean([f[1] for f in flops]))
    attn_avg_ms = float(attn_ms.mean())
    achieved = useful_flop / (attn_avg_ms * 1e-3) / 1e12

    elt = 2 if bf16 else 4
    bt = tile_t * w.tile_h * w.tile_w
    tok_new = w.q_frames * w.tokens_per_frame
    # append traffic (algorithmic): read new K,V once, write their tiles once, write pooled K
    append_bytes = 2 * tok_new * g.heads * g.head_dim * elt + 2 * n_qb * bt * g.head_dim * elt * g.heads \
        + n_qb * g.heads * g.head_dim * 4
    pool_bytes = tok_new * g.heads * g.head_dim * elt + n_qb * g.heads * g.head_dim * 4
    # selection: pooled Q and the pooled K of every visible block once, ids + counts out
    select_bytes = (n_qb + w.cache_frames // tile_t * g.nb) * g.heads * g.head_dim * 4 + g.heads * n_qb * (topk + 1) * 4
    mfma_path = bf16 and g.head_dim == 128 and bt == 128
    peak = PEAK_BF16_TFLOPS if mfma_path else PEAK_F32_TFLOPS
    plain = not (args.blocks or args.grid or args.cache_frames) and args.radius is None and policy == B.LCSA_EVICT_SLIDING
    res = {
        "ms_per_layer": ms_per_layer, "ms_per_step": ms_per_step,
        "config": {"workload": WORKLOAD_TEXT[name], "heads": g.heads, "head_dim": g.head_dim,
                   "layers_per_step": n_layers, "q_tokens": tok_new, "kv_tokens": w.cache_frames * w.tokens_per_frame,
                   "block_shape": [tile_t, w.tile_h, w.tile_w], "blocks_per_group": g.nb, "query_blocks": n_qb,
                   "grid": [w.grid_h, w.grid_w], "cache_frames": w.cache_frames, "topk": topk, "radius": radius,
                   "eviction": args.eviction, "launch": "hip graphs" if args.graph else "eager"},
        **({"hip_graph_replay_ms_per_chunk_per_layer": round(replay_ms_per_layer, 5)} if replay_ms_per_layer else {}),
        "effective_tflops_whole_path": round(useful_flop / (ms_per_layer * 1e-3) / 1e12, 2),
        "kernel_ms_per_layer": {"kv_cache_append": round(float(brk[0]), 5),
                                **({"pool_blocks": round(float(brk[1]), 5), "select_blocks": round(float(brk[2]), 5)}
                                   if args.two_calls else {"pool_select_blocks": round(float(brk[2]), 5)}),
                                "sparse_attn_fwd": round(attn_avg_ms, 5),
                                **({"block_importance": round(float(brk[4]), 5)} if scoring else {})},
        "hbm_gbs": {"kv_cache_append": round(append_bytes / (brk[0] * 1e-3) / 1e9, 1),
                    **({"pool_blocks": round(pool_bytes / (brk[1] * 1e-3) / 1e9, 1),
                        "select_blocks": round(select_bytes / (brk[2] * 1e-3) / 1e9, 1)} if args.two_calls else
                       {"pool_select_blocks": round((pool_bytes + select_bytes) / (brk[2] * 1e-3) / 1e9, 1)})},
        "roofline": {"kernel": "attn_mfma_kernel" if mfma_path else "attn_generic_kernel",
                     "bound": "mfma" if mfma_path else "alu", "achieved": round(achieved, 3),
                     "peak": peak, "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
                     "traffic": attn_traffic_from_profiles(name, topk) if plain and mfma_path else None,
                     "flop_per_launch_useful": useful_flop, "flop_per_launch_issued": issued_flop,
                     "issued_tflops": round(issued_flop / (attn_avg_ms * 1e-3) / 1e12, 3),
                     "avg_launch_ms": round(attn_avg_ms, 5), "min_launch_ms": round(float(attn_ms.min()), 5)},
        "setup_s": round(setup_s, 1),
    }
    live = dict(w=w, g=g, layers=layers, host_layer0=host_layer0, gen=gen, tile_t=tile_t, radius=radius, topk=topk,
                n_layers=n_layers, dev=dev, mfma_path=mfma_path)
    return res, live


def streaming_sweep(torch, B, wl, live, topks=(16, 32, 64)):
    """One video from an empty cache, chunk by chunk, for several top-k values: per-chunk time of the whole path
    while the ring fills and in the steady state (attention launches timed separately)."""
    w, g0, dev, tile_t, radius = live["w"], live["g"], live["dev"], live["tile_t"], live["radius"]
    s0 = wl.ChunkStream(w, 0)
    vchunks = [tuple(dev(x) for x in s0.next()) for _ in range(w.n_chunks)]
    fill = (w.cache_frames - w.q_frames) // w.q_frames           # chunks before the ring is full
    n_qb = g0.n_qb
    valid_tok = valid_tokens_per_block(w, tile_t)
    out = {}
    for rep, k in enumerate((topks[0],) + tuple(topks)):              # the first pass only warms up
        gk = B.Geom(w.heads, w.head_dim, w.grid_h, w.grid_w, w.tile_h, w.tile_w, w.q_frames, w.cache_frames,
                    radius, radius, k, dtype=g0.dtype, tile_t=tile_t)
        cache = B.lcsa_cache_init(gk)
        pq = torch.empty(gk.heads, n_qb, gk.head_dim, dtype=torch.float32, device="cuda")
        si = torch.empty(gk.heads, n_qb, k, dtype=torch.int32, device="cuda")
        sc = torch.empty(gk.heads, n_qb, dtype=torch.int32, device="cuda")
        oo = torch.empty_like(vchunks[0][0])
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(len(vchunks) + 1)]
        aev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in vchunks]
        torch.cuda.synchronize()
        evs[0].record()
        for i, (qd, kd, vd) in enumerate(vchunks):
            B.lcsa_kv_cache_append(cache, kd, vd, w.q_frames)
            B.lcsa_pool_select_blocks(gk, qd, cache, pq, si, sc, want_gap=False)
            aev[i][0].record()
            B.lcsa_sparse_attn_fwd(gk, qd, cache, si, sc, oo)
            aev[i][1].record()
            evs[i + 1].record()
        torch.cuda.synchronize()
        ms = [evs[i].elapsed_time(evs[i + 1]) for i in range(len(vchunks))]
        ams = [a.elapsed_time(b) for a, b in aev]
        if rep:
            flop, _ = attention_flop(si, valid_tok, n_qb, gk.nb, gk.head_dim)      # a steady-state launch: the last selection
            steady_attn = float(np.mean(ams[fill:]))
            out[f"topk_{k}"] = {"ring_filling_ms_per_chunk": [round(x, 4) for x in ms[:fill]],
                                "steady_ms_per_chunk_mean": round(float(np.mean(ms[fill:])), 4),
                                "steady_ms_per_chunk_min": round(float(np.min(ms[fill:])), 4),
                                "steady_attn_ms": round(steady_attn, 4),
                                "steady_attn_tflops": round(flop / (steady_attn * 1e-3) / 1e12, 1),
                                "steady_attn_roofline_frac": round(flop / (steady_attn * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)}
        del cache, pq, si, sc, oo
    return {"chunks": len(vchunks), "chunks_before_ring_is_full": fill, **out}


def attn_timers(torch, B, aids, live):
    """Time stamps of every workgroup of one attention launch (layer 0 of the workload as it stands): shader clock
    under load and time per workgroup, for the workgroups that start with the launch (one per compute unit) and
    for those that start later (on fewer busy compute units).  Stamps inside the kernel (before and after the
    main loop, -DLCSA_TIMERS=1) slow its loop by 16 %, so the aid is built with entry and exit stamps only."""
    g, L = live["g"], live["layers"][0]
    q = L["chunks"][(L["turn"] - 1) % len(L["chunks"])][0]
    total = g.heads * g.n_qb
    n_wg = 8 * -(-((total + 1) // 2) // 8)
    stamps = torch.zeros(n_wg, 10, dtype=torch.int64, device="cuda")
    gc = g.c()
    cnt = L["sel_cnt"].cpu().numpy()
    for _ in range(3):                                   # the last of three launches is read (the first ones warm up)
        stamps.zero_()
        rc = aids.lib.bench_attn_timed(ctypes.byref(gc), q.data_ptr(), q.stride(0), q.stride(1), L["cache"].handle,
                                       L["sel_idx"].data_ptr(), L["sel_cnt"].data_ptr(), L["o"].data_ptr(),
                                       L["o"].stride(0), L["o"].stride(1), 0.0, stamps.data_ptr(),
                                       torch.cuda.current_stream().cuda_stream)
        if rc != 0:
            return None
        torch.cuda.synchronize()
    t = stamps.cpu().numpy().astype(np.float64)
    t = t[t[:, 0] > 0]
    if len(t) == 0:
        return None
    clk = lambda a, b: (t[:, 2 * b] - t[:, 2 * a])                    # shader cycles between stamps a and b
    wall = lambda a, b: (t[:, 2 * b + 1] - t[:, 2 * a + 1]) * 10.0     # ns (100 MHz counter)
    steps = int(cnt.max()) + 1                                         # loop iterations of a full workgroup
    start_ns = (t[:, 1] - t[:, 1].min()) * 10.0
    first = start_ns < 0.25 * wall(0, 3).mean()                        # workgroups that started with the launch

    def rnd(sel):
        if sel.sum() == 0:
            return None
        return {"workgroups": int(sel.sum()),
                "shader_clock_ghz": round(float(clk(0, 3)[sel].sum() / wall(0, 3)[sel].sum()), 3),
                "us_per_workgroup": round(float(np.median(wall(0, 3)[sel])) / 1e3, 2),
                "shader_cycles_per_workgroup": round(float(np.median(clk(0, 3)[sel]))),
                "shader_cycles_per_loop_step_incl_setup_and_epilogue": round(float(np.median(clk(0, 3)[sel])) / steps, 1)}

    span = (t[:, 7].max() - t[:, 1].min()) * 10.0
    return {"kernel": "attn_mfma_kernel built with -DLCSA_TIMERS=2 (libbench_probe.so): stamps at entry and exit of every workgroup",
            "workgroups_that_ran": int(len(t)), "loop_steps_per_workgroup": steps,
            "matrix_cycles_per_loop_step_per_simd": 4096,
            "first_stamp_to_last_stamp_us": round(float(span) / 1e3, 2),
            "started_with_the_launch": rnd(first), "started_later": rnd(~first)}


def trivial_loops(torch, aids):
    """What this chip sustains on trivial loops, quoted beside the nominal peaks."""
    prop = torch.cuda.get_device_properties(0)
    n_cu = prop.multi_processor_count
    pe = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    cur = torch.cuda.current_stream().cuda_stream
    out = {"mfma_bf16_register_loop_tflops": None, "mock_inner_loop_tflops": None}
    if aids.lib:
        buf = torch.empty(n_cu * 2 * 512, dtype=torch.float32, device="cuda")
        iters = 4000
        assert aids.lib.bench_probe_mfma_bf16(buf.data_ptr(), n_cu * 2, 200, cur) == 0
        pe[0].record()
        assert aids.lib.bench_probe_mfma_bf16(buf.data_ptr(), n_cu * 2, iters, cur) == 0
        pe[1].record()
        torch.cuda.synchronize()
        out["mfma_bf16_register_loop_tflops"] = round(n_cu * 2 * 8 * iters * 32 * 32768.0 / (pe[0].elapsed_time(pe[1]) * 1e-3) / 1e12, 1)
        src = torch.ones(16 << 20, dtype=torch.uint8, device="cuda")
        mock = {}
        for variant, label in ((0, "mfma+lds_operands"), (1, "+4_valu_per_mfma"), (2, "+barrier_per_32_mfma"),
                               (3, "+tile_copies (the full mix)"), (4, "the full mix with 5 valu"),
                               (5, "the full mix without mfma: ns per step")):
            steps = 3000
            assert aids.lib.bench_mock_loop(variant, buf.data_ptr(), src.data_ptr(), n_cu, 50, cur) == 0
            pe[0].record()
            assert aids.lib.bench_mock_loop(variant, buf.data_ptr(), src.data_ptr(), n_cu, steps, cur) == 0
            pe[1].record()
            torch.cuda.synchronize()
            ms = pe[0].elapsed_time(pe[1])
            mock[label] = round(ms * 1e6 / steps, 1) if variant == 5 else round(n_cu * 8 * 32 * 32768.0 * steps / (ms * 1e-3) / 1e12, 1)
        out["mock_inner_loop_tflops"] = mock
        del buf, src
    csrc = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
    cdst = torch.empty_like(csrc)
    cdst.copy_(csrc)
    pe[0].record()
    for _ in range(5):
        cdst.copy_(csrc)
    pe[1].record()
    torch.cuda.synchronize()
    out["device_copy_gbs"] = round(5 * 2 * float(1 << 30) / (pe[0].elapsed_time(pe[1]) * 1e-3) / 1e9, 1)
    # the same copy at the size of one paper-scale append (52 MB in, 52 MB out), over 16 different slices in turn so
    # that neither side stays in the 256 MB Infinity Cache: what a launch of that size reaches from HBM
    n_small = 52 << 20
    sl = lambda t, i: t[(i % 16) * n_small:(i % 16 + 1) * n_small]
    for i in range(4):
        sl(cdst, i).copy_(sl(csrc, i + 5))
    pe[0].record()
    for i in range(32):
        sl(cdst, i).copy_(sl(csrc, i + 5))
    pe[1].record()
    torch.cuda.synchronize()
    out["device_copy_52MB_us"] = round(pe[0].elapsed_time(pe[1]) * 1e3 / 32, 2)
    out["device_copy_52MB_gbs"] = round(32 * 2 * float(n_small) / (pe[0].elapsed_time(pe[1]) * 1e-3) / 1e9, 1)
    del csrc, cdst
    return out, prop, n_cu


def extensions(torch, B, wl):
    """The calls beside the forward path, timed briefly: the backward of the attention (matrix-core kernels at
    small-video and paper scale, the float FMA kernels at small-video scale) and the fused rotary embedding +
    pooling of a paper-scale chunk's queries (bound by HBM)."""
    out = {}
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    dev = lambda x: torch.from_numpy(wl.bf16_bits(x).view(np.int16)).view(torch.bfloat16).cuda()
    for name in ("small", "paper"):
        w = wl.WORKLOADS[name]
        g = B.Geom(w.heads, w.head_dim, w.grid_h, w.grid_w, w.tile_h, w.tile_w, w.q_frames, w.cache_frames, w.radius, w.radius,
                   w.topk, dtype=B.LCSA_BF16)
        s = wl.ChunkStream(w, 0)
        chunks = [s.next() for _ in range(w.prime_chunks + 1)]
        cache = B.lcsa_cache_init(g)
        for (_, k, v) in chunks:
            B.lcsa_kv_cache_append(cache, dev(k), dev(v), w.q_frames)
        qd = dev(chunks[-1][0])
        K = dev(np.concatenate([c[1] for c in chunks]))
        V = dev(np.concatenate([c[2] for c in chunks]))
        _, si, sc, _ = B.lcsa_pool_select_blocks(g, qd, cache, want_gap=False)
        lse = torch.empty(qd.shape[0], g.heads, dtype=torch.float32, device="cuda")
        B.lcsa_sparse_attn_fwd(g, qd, cache, si, sc, lse=lse)
        d_o = torch.randn_like(qd)
        fwd_flop, fwd_issued = attention_flop(si, valid_tokens_per_block(w, 1), g.n_qb, g.nb, g.head_dim)
        for float_path in ((False, True) if name == "small" else (False,)):
            reps = 3 if float_path else 20
            for _ in range(2):
                B.lcsa_sparse_attn_bwd(g, qd, K, V, w.cache_frames, si, sc, d_o, lse, float_path=float_path)
            ev[0].record()
            for _ in range(reps):
                B.lcsa_sparse_attn_bwd(g, qd, K, V, w.cache_frames, si, sc, d_o, lse, float_path=float_path)
            ev[1].record()
            torch.cuda.synchronize()
            ms = ev[0].elapsed_time(ev[1]) / reps
            # five products where the forward has two (useful: 2.5 x); the kernels execute nine (q.k and dO.v are formed
            # in the pass that yields D, in the dQ pass and in the dK/dV pass): 4.5 x the forward's executed flop
            useful, executed = 2.5 * fwd_flop, 4.5 * fwd_issued
            peak = PEAK_F32_TFLOPS if float_path else PEAK_BF16_TFLOPS
            out[f"sparse_attn_bwd_{name}_{'float' if float_path else 'matrix_cores'}"] = {
                "ms": round(ms, 4), "flop_useful": useful, "flop_executed": executed,
                "useful_tflops": round(useful / (ms * 1e-3) / 1e12, 2),
                "roofline": {"bound": "alu" if float_path else "mfma", "achieved": round(executed / (ms * 1e-3) / 1e12, 2),
                             "peak": peak, "unit": "TFLOP/s", "frac": round(executed / (ms * 1e-3) / 1e12 / peak, 4)}}
        del cache, K, V
    # ---- rotary embedding + pooling, the queries of a paper-scale chunk
    w = wl.WORKLOADS["paper"]
    g = B.Geom(w.heads, w.head_dim, w.grid_h, w.grid_w, w.tile_h, w.tile_w, w.q_frames, w.cache_frames, w.radius, w.radius,
               w.topk, dtype=B.LCSA_BF16)
    x = torch.randn(w.q_frames * w.tokens_per_frame, w.heads, w.head_dim, device="cuda").to(torch.bfloat16)
    xr = torch.empty_like(x)
    pooled = torch.empty(g.heads, g.n_qb, g.head_dim, dtype=torch.float32, device="cuda")
    third = g.head_dim // 6
    pairs = (g.head_dim // 2 - 2 * third, third, third)
    for _ in range(3):
        B.lcsa_rope_pool_blocks(g, x, w.q_frames, pairs, 0.0, 7, xr, pooled)
    ev[0].record()
    for _ in range(20):
        B.lcsa_rope_pool_blocks(g, x, w.q_frames, pairs, 0.0, 7, xr, pooled)
    ev[1].record()
    torch.cuda.synchronize()
    ms = ev[0].elapsed_time(ev[1]) / 20
    nbytes = 2 * x.numel() * 2 + pooled.numel() * 4
    out["rope_pool_blocks_paper_q"] = {"ms": round(ms, 5), "bytes": nbytes, "gbs": round(nbytes / (ms * 1e-3) / 1e9, 1),
                                       "roofline": {"bound": "hbm", "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                                    "frac": round(nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}}
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="paper", choices=sorted(WORKLOAD_TEXT))
    ap.add_argument("--layers", type=int, default=0, help="override the workload's number of layer calls")
    ap.add_argument("--topk", type=int, default=0, help="override top-k (a value >= the window size gives windowed dense attention)")
    ap.add_argument("--radius", type=int, default=None, help="override the locality radius in tokens (-1: unbounded window)")
    ap.add_argument("--blocks", default="", help="block shape t,h,w overriding the workload's 1,tile_h,tile_w (e.g. 2,8,8: the paper's partition)")
    ap.add_argument("--grid", default="", help="latent grid h,w overriding the workload's (e.g. 96,168: a 1536x2688 video)")
    ap.add_argument("--cache-frames", type=int, default=0, help="override the sliding-window capacity in frames")
    ap.add_argument("--eviction", default="sliding", choices=["sliding", "headwise", "uniform"],
                    help="KV-cache eviction: the paper's default sliding window, or importance-based (adds lcsa_block_importance to every layer call)")
    ap.add_argument("--graph-too", action="store_true", help=argparse.SUPPRESS)   # set for the headline workload of a default run
    ap.add_argument("--graph", action="store_true",
                    help="replay the layer calls of a step from captured HIP graphs (the caches are full when they are recorded)")
    ap.add_argument("--two-calls", action="store_true",
                    help="pool and select with lcsa_pool_blocks + lcsa_select_blocks instead of the fused lcsa_pool_select_blocks")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="skip the short measurements of the other benchmark configurations")
    ap.add_argument("--no-streaming", action="store_true", help="skip the chunk-by-chunk stream with its top-k sweep (4k workload)")
    ap.add_argument("--only-extensions", action="store_true", help="time only the calls beside the forward path (backward, fused rotary embedding + pooling)")
    ap.add_argument("--no-aids", action="store_true", help="skip the trivial-loop rates and the kernel time stamps")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device-to-device copy first (reference point for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures ONE GPU (the path has no inter-GPU part); run with --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2510_12747_amd import binding as B
    from paper_2510_12747_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    B.lib()   # fail loudly if the HIP library is not built
    aids = Aids()

    if args.only_extensions:
        print(json.dumps({"extensions": extensions(torch, B, wl)}))
        return 0

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    args.graph_too = not args.graph and not args.no_others        # a default run also replays the step from captured graphs
    res, live = measure(torch, B, wl, args, args.workload, args.steps, args.warmup)
    args.graph_too = False
    w = live["w"]
    out = {
        "metric": "sparse_attn_ms_per_chunk_per_layer",
        "value": round(res["ms_per_layer"], 5),
        "unit": "ms",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(res["ms_per_step"], 4),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        # element type of Q, K, V, O and of the first matrix product; the second product takes probabilities and V
        # as IEEE half (same matrix rate); every accumulation and the softmax are float
        "dtype": "bf16" if w.dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": res["config"],
        "effective_tflops_whole_path": res["effective_tflops_whole_path"],
        "kernel_ms_per_layer": res["kernel_ms_per_layer"],
        "hbm_gbs": res["hbm_gbs"],
        "roofline": res["roofline"],
        "setup_s": res["setup_s"],
    }
    if "hip_graph_replay_ms_per_chunk_per_layer" in res:      # same step, replayed from captured HIP graphs: beside `value`, not it
        out["hip_graph_replay_ms_per_chunk_per_layer"] = res["hip_graph_replay_ms_per_chunk_per_layer"]
    if w.n_chunks > 1 and not args.no_streaming:
        out["streaming"] = streaming_sweep(torch, B, wl, live)

    if not args.no_aids:
        if aids.lib and live["mfma_path"]:      # first: right after the timed region, in the same thermal state
            out["attn_timers"] = attn_timers(torch, B, aids, live)
        peaks, prop, n_cu = trivial_loops(torch, aids)
        out["device"] = {"name": prop.name, "compute_units": n_cu, "nominal_peak_tflops": PEAK_BF16_TFLOPS,
                         "nominal_hbm_gbs": PEAK_HBM_GBS}
        out["measured_peaks"] = peaks
        if peaks["mfma_bf16_register_loop_tflops"]:
            out["roofline"]["frac_of_measured_mfma_loop"] = round(out["roofline"]["achieved"] / peaks["mfma_bf16_register_loop_tflops"], 4)

    # ---- CPU oracle on the host cores: a bounded sample of the same workload ------------------------
    # Whole layer calls (pooling, scores, selection, attention of every row) of the first layers of
    # the workload, as many as fit in about 15 s (at least one, at most five); value = mean per layer.
    if not args.no_cpu_baseline:
        import oracle
        og = oracle.Geometry(w.heads, w.head_dim, w.grid_h, w.grid_w, w.tile_h, w.tile_w, w.q_frames,
                             live["radius"], live["radius"], live["topk"], tile_t=live["tile_t"])
        times = []
        for layer in range(min(5, live["n_layers"])):
            chunks = live["host_layer0"] if layer == 0 else live["gen"](layer)
            model = oracle.SlidingWindowCache(w.cache_frames)
            for (q, k, v) in chunks:
                model.append(k, v, w.q_frames)
            K, V = model.visible()
            t1 = time.perf_counter()
            oracle.lcsa(chunks[-1][0], K, V, og, model.valid_frames)
            times.append(time.perf_counter() - t1)
            if sum(times) > 15.0:
                break
        out["cpu_baseline"] = {"value": round(float(np.mean(times)) * 1e3, 1), "unit": "ms", "cores": oracle.threads(),
                               "kind": "oracle",
                               "sample": f"{len(times)} of {live['n_layers']} layer calls of the same workload, each in full "
                                         f"(pool, scores, select, attend all rows); {sum(times):.1f} s of CPU time; "
                                         f"value = mean ms per chunk per layer"}
    del live, res

    # ---- the other benchmark configurations, briefly (outside the timed region of the headline) -------------
    if not args.no_others and not (args.blocks or args.grid or args.cache_frames or args.topk or args.layers
                                   or args.radius is not None):
        others = {}
        for name in ("tiny", "small", "paper", "ultra", "4k"):
            if name == args.workload:
                continue
            torch.cuda.empty_cache()
            # 4 layer calls per step, 4 warm-up and 10 timed steps: shorter runs are dominated by the ramp of the
            # clocks and read 20 % slow
            r, lv = measure(torch, B, wl, args, name, steps=10, warmup=4, n_layers=4)
            entry = {"ms_per_chunk_per_layer": round(r["ms_per_layer"], 5), "kernel_ms_per_layer": r["kernel_ms_per_layer"],
                     "hbm_gbs": r["hbm_gbs"],
                     "roofline": {k: r["roofline"][k] for k in ("kernel", "bound", "achieved", "peak", "unit", "frac", "traffic", "avg_launch_ms")},
                     "layers_per_step": 4, "steps": 10, "warmup": 4}
            if lv["w"].n_chunks > 1:
                entry["streaming"] = streaming_sweep(torch, B, wl, lv)
            others[name] = entry
            del lv, r
        out["other_workloads"] = others
        torch.cuda.empty_cache()
        out["extensions"] = extensions(torch, B, wl)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
