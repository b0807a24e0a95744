#!/usr/bin/env python3
"""Benchmark of the locality-constrained block-sparse attention hot path on one MI355X.

One STEP = one chunk of latent frames through every layer of the workload: per layer
lcsa_kv_cache_append -> lcsa_pool_blocks -> lcsa_select_blocks -> lcsa_sparse_attn_fwd, each
layer with its own seeded Q/K/V and its own sliding-window cache (already primed, so the timed
step runs in steady state: append evicts the oldest frames, attention sees a full window).
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload paper|small|ultra|4k]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 / fp16 matrix peak
PEAK_HBM_GBS = 8000.0

# HBM-side bytes per attention launch (L2 <-> fabric), from the rocprofv3 --pmc passes summarised in
# profiles/hot_path_paper_scale_pmc.txt: FETCH_SIZE x 2.0 (factor from a 1 GiB copy) + WRITE_SIZE x 1.0, in bytes.
# Counters cannot be read from inside this script; the figure is only quoted for the workload it was taken on.
ATTN_TRAFFIC_BYTES = {("paper", 32): 278.9e6 + 25.9e6}

WORKLOAD_TEXT = {
    "paper": "paper-scale 768x1408: 48x88 tokens/frame, 2 query + 4 cached frames, 8x16 tiles, radius 24, top-k 32, 30 layer calls",
    "small": "small-video 384x704: 24x44 tokens/frame, 2 query + 4 cached frames, 8x16 tiles, radius 16, top-k 16",
    "ultra": "ultra-high-res 1440x2560: 90x160 tokens/frame, 2 query + 4 cached frames, 8x16 tiles, radius 24, top-k 32",
    "4k": "4k streaming 2160x3840: 135x240 tokens/frame, 1 query frame, ring of 6 frames, 8x16 tiles, radius 24, top-k 32",
}


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
    ap.add_argument("--graph", action="store_true",
                    help="replay the layer calls of a step from captured HIP graphs (the caches are full when they are recorded)")
    ap.add_argument("--two-calls", action="store_true",
                    help="pool and select with lcsa_pool_blocks + lcsa_select_blocks instead of the fused lcsa_pool_select_blocks")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device-to-device copy (reference point for HBM byte counters)")
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

    w = wl.WORKLOADS[args.workload]
    n_layers = args.layers or w.n_layers
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
    g = B.Geom(w.heads, w.head_dim, w.grid_h, w.grid_w, w.tile_h, w.tile_w, w.q_frames, w.cache_frames,
               radius, radius, topk, dtype=B.LCSA_BF16, tile_t=tile_t)
    n_qb = g.n_qb
    policy = {"sliding": B.LCSA_EVICT_SLIDING, "headwise": B.LCSA_EVICT_IMPORTANCE_HEADWISE,
              "uniform": B.LCSA_EVICT_IMPORTANCE_UNIFORM}[args.eviction]
    scoring = policy != B.LCSA_EVICT_SLIDING

    def dev(x):
        return torch.from_numpy(wl.bf16_bits(x).view(np.int16)).view(torch.bfloat16).cuda()

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

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        for L in layers:
            layer_call(L)
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps; HIP events around every attention launch ------------------
    # (all launches go to torch's current stream, which is the stream these events are recorded on)
    attn_ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in layers]
               for _ in range(args.steps)]
    graphs = []
    if args.graph:
        # one graph per position of the chunk rotation: the inputs of a captured call are fixed
        for _ in range(len(layers[0]["chunks"])):
            gph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gph):
                for L in layers:
                    layer_call(L)
            graphs.append(gph)
        for s_ in range(args.warmup):
            graphs[s_ % len(graphs)].replay()
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for s in range(args.steps):
        if args.graph:
            graphs[(args.warmup + s) % len(graphs)].replay()
        else:
            for L, (e0, e1) in zip(layers, attn_ev[s]):
                layer_call(L, attn_ev=(e0, e1))
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    ms_per_step = elapsed * 1e3 / args.steps
    ms_per_layer = ms_per_step / n_layers
    attn_ms = None if args.graph else np.array([[e0.elapsed_time(e1) for (e0, e1) in step] for step in attn_ev])

    # ---- untimed breakdown pass: events between the four calls ------------------------------------
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in layers]
    for L, e in zip(layers, ev):
        e[4].record()
        layer_call(L, e)
    torch.cuda.synchronize()
    brk = np.array([[e[4].elapsed_time(e[0]), e[0].elapsed_time(e[1]), e[1].elapsed_time(e[2]), e[2].elapsed_time(e[3]),
                     e[3].elapsed_time(e[5])] for e in ev]).mean(axis=0)
    if attn_ms is None:      # launches inside a graph carry no events: the attention launches of this eager pass stand in
        attn_ms = np.array([[e[2].elapsed_time(e[3]) for e in ev]])

    # ---- what this chip sustains on trivial loops, quoted beside the nominal peaks (outside the timed region):
    # back-to-back bf16 matrix instructions on registers, and a 1 GiB device-to-device copy
    prop = torch.cuda.get_device_properties(0)
    n_cu = prop.multi_processor_count
    pe = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    probe_tflops = None
    probe_path = os.path.join(ROOT, "libbench_probe.so")      # bench-only shared object, built by __graft_entry__.build()
    if os.path.exists(probe_path):
        import ctypes
        probe = ctypes.CDLL(probe_path).bench_probe_mfma_bf16
        probe.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p]
        probe.restype = ctypes.c_int32
        probe_out = torch.empty(n_cu * 2 * 512, dtype=torch.float32, device="cuda")
        probe_iters = 4000
        cur = torch.cuda.current_stream().cuda_stream
        assert probe(probe_out.data_ptr(), n_cu * 2, 200, cur) == 0
        pe[0].record()
        assert probe(probe_out.data_ptr(), n_cu * 2, probe_iters, cur) == 0
        pe[1].record()
        torch.cuda.synchronize()
        probe_tflops = n_cu * 2 * 8 * probe_iters * 32 * 32768.0 / (pe[0].elapsed_time(pe[1]) * 1e-3) / 1e12
        del probe_out
    csrc = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
    cdst = torch.empty_like(csrc)
    cdst.copy_(csrc)
    pe[0].record()
    for _ in range(5):
        cdst.copy_(csrc)
    pe[1].record()
    torch.cuda.synchronize()
    copy_gbs = 5 * 2 * float(1 << 30) / (pe[0].elapsed_time(pe[1]) * 1e-3) / 1e9
    del csrc, cdst

    # ---- algorithmic work of one attention launch (from the selection actually made) ---------------
    ty, tx = -(-w.grid_h // w.tile_h), -(-w.grid_w // w.tile_w)
    vh = np.minimum(w.tile_h, w.grid_h - np.arange(ty) * w.tile_h)
    vw = np.minimum(w.tile_w, w.grid_w - np.arange(tx) * w.tile_w)
    valid_tok = (vh[:, None] * vw[None, :]).reshape(-1) * tile_t     # valid tokens per block
    useful, issued = [], []
    for L in layers:
        idx = L["sel_idx"].cpu().numpy()
        cnt = L["sel_cnt"].cpu().numpy()
        kvalid = np.where(idx >= 0, valid_tok[np.maximum(idx, 0) % g.nb], 0).sum(axis=-1)   # [h][qb]
        qvalid = valid_tok[np.arange(n_qb) % g.nb][None, :]
        useful.append(4.0 * g.head_dim * float((qvalid * kvalid).sum()))
        # the kernel computes whole 32-query x 32-key matrix-core tiles: valid counts rounded up to 32
        up32 = -(-valid_tok // 32) * 32
        kiss = np.where(idx >= 0, up32[np.maximum(idx, 0) % g.nb], 0).sum(axis=-1)
        qiss = up32[np.arange(n_qb) % g.nb][None, :]
        issued.append(4.0 * g.head_dim * float((qiss * kiss).sum()))
    useful_flop, issued_flop = float(np.mean(useful)), float(np.mean(issued))
    attn_avg_ms = float(attn_ms.mean())
    achieved = useful_flop / (attn_avg_ms * 1e-3) / 1e12

    # append traffic (algorithmic): read new K,V once, write their tiles once, write pooled K
    tok_new = w.q_frames * w.tokens_per_frame
    append_bytes = 2 * tok_new * g.heads * g.head_dim * 2 + 2 * n_qb * 128 * 128 * 2 * g.heads \
        + n_qb * g.heads * g.head_dim * 4
    pool_bytes = tok_new * g.heads * g.head_dim * 2 + n_qb * g.heads * g.head_dim * 4
    # selection: pooled Q and the pooled K of every visible block once, ids + counts out
    select_bytes = (n_qb + w.cache_frames // tile_t * g.nb) * g.heads * g.head_dim * 4 + g.heads * n_qb * (topk + 1) * 4

    out = {
        "metric": "sparse_attn_ms_per_chunk_per_layer",
        "value": round(ms_per_layer, 5),
        "unit": "ms",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT[args.workload], "heads": g.heads, "head_dim": g.head_dim,
                   "layers_per_step": n_layers, "q_tokens": tok_new, "kv_tokens": w.cache_frames * w.tokens_per_frame,
                   "block_shape": [tile_t, w.tile_h, w.tile_w], "blocks_per_group": g.nb, "query_blocks": n_qb,
                   "grid": [w.grid_h, w.grid_w], "cache_frames": w.cache_frames, "topk": topk, "radius": radius,
                   "eviction": args.eviction, "launch": "hip graphs" if args.graph else "eager"},
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
        "device": {"name": prop.name, "compute_units": n_cu,
                   "nominal_peak_tflops": PEAK_BF16_TFLOPS, "nominal_hbm_gbs": 8000.0},
        "measured_peaks": {"mfma_bf16_register_loop_tflops": round(probe_tflops, 1) if probe_tflops else None,
                           "device_copy_gbs": round(copy_gbs, 1)},
        "roofline": {"kernel": "attn_mfma_kernel", "bound": "mfma", "achieved": round(achieved, 2),
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                     "traffic": ATTN_TRAFFIC_BYTES.get((args.workload, topk)) if not (args.blocks or args.grid or args.cache_frames) and args.radius is None and policy == B.LCSA_EVICT_SLIDING else None,
                     "flop_per_launch_useful": useful_flop, "flop_per_launch_issued": issued_flop,
                     "issued_tflops": round(issued_flop / (attn_avg_ms * 1e-3) / 1e12, 2),
                     "avg_launch_ms": round(attn_avg_ms, 5), "min_launch_ms": round(float(attn_ms.min()), 5),
                     # beside the nominal peak: the same figure against what a register-only MFMA loop sustains here
                     "frac_of_measured_mfma_loop": round(achieved / probe_tflops, 4) if probe_tflops else None},
        "setup_s": round(setup_s, 1),
    }

    # ---- streaming workloads: one video from an empty cache, chunk by chunk, for three top-k values -----
    # (per-chunk time of the whole path while the ring fills and in the steady state; outside the timed region)
    if w.n_chunks > 1:
        s0 = wl.ChunkStream(w, 0)
        vchunks = [tuple(dev(x) for x in s0.next()) for _ in range(w.n_chunks)]
        fill = (w.cache_frames - w.q_frames) // w.q_frames           # chunks before the ring is full
        streaming = {}
        for rep, k in enumerate((topk, 16, 32, 64)):                  # the first pass only warms up
            gk = B.Geom(w.heads, w.head_dim, w.grid_h, w.grid_w, w.tile_h, w.tile_w, w.q_frames, w.cache_frames,
                        radius, radius, k, dtype=B.LCSA_BF16, tile_t=tile_t)
            cache = B.lcsa_cache_init(gk)
            pq = torch.empty(gk.heads, n_qb, gk.head_dim, dtype=torch.float32, device="cuda")
            si = torch.empty(gk.heads, n_qb, k, dtype=torch.int32, device="cuda")
            sc = torch.empty(gk.heads, n_qb, dtype=torch.int32, device="cuda")
            oo = torch.empty_like(vchunks[0][0])
            evs = [torch.cuda.Event(enable_timing=True) for _ in range(len(vchunks) + 1)]
            torch.cuda.synchronize()
            evs[0].record()
            for i, (qd, kd, vd) in enumerate(vchunks):
                B.lcsa_kv_cache_append(cache, kd, vd, w.q_frames)
                B.lcsa_pool_blocks(gk, qd, w.q_frames, pq)
                B.lcsa_select_blocks(gk, pq, cache, si, sc, want_gap=False)
                B.lcsa_sparse_attn_fwd(gk, qd, cache, si, sc, oo)
                evs[i + 1].record()
            torch.cuda.synchronize()
            ms = [evs[i].elapsed_time(evs[i + 1]) for i in range(len(vchunks))]
            if rep:
                streaming[f"topk_{k}"] = {"ring_filling_ms_per_chunk": [round(x, 4) for x in ms[:fill]],
                                          "steady_ms_per_chunk_mean": round(float(np.mean(ms[fill:])), 4),
                                          "steady_ms_per_chunk_min": round(float(np.min(ms[fill:])), 4)}
            del cache, pq, si, sc, oo
        out["streaming"] = {"chunks": len(vchunks), "chunks_before_ring_is_full": fill, **streaming}
        del vchunks

    # ---- CPU oracle on the host cores: a bounded sample of the same workload ------------------------
    # Whole layer calls (pooling, scores, selection, attention of every row) of the first layers of
    # the workload, as many as fit in about 15 s (at least one, at most five); value = mean per layer.
    if not args.no_cpu_baseline:
        import oracle
        og = oracle.Geometry(w.heads, w.head_dim, w.grid_h, w.grid_w, w.tile_h, w.tile_w, w.q_frames,
                             radius, radius, topk, tile_t=tile_t)
        times = []
        for layer in range(min(5, n_layers)):
            chunks = host_layer0 if layer == 0 else gen(layer)
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
                               "sample": f"{len(times)} of {n_layers} layer calls of the same workload, each in full "
                                         f"(pool, scores, select, attend all rows); {sum(times):.1f} s of CPU time; "
                                         f"value = mean ms per chunk per layer"}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
