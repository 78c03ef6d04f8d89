#!/usr/bin/env python3
"""Benchmark of the KVCrush per-layer compression step on one MI355X.

A step is one pass of the whole hot path over one layer of the workload:
row normalisers (pass A) -> received-attention scores (pass B) -> selection
(top-k, bits, Hamming grouping, representatives) -> K/V gather.  The layers'
Q/K/V are generated once and stay resident in HBM; successive steps walk
through the layers so that the 256 MB last-level cache cannot serve repeats.

Prints ONE JSON line (the last line of stdout).
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

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 matrix peak, vendor figure
HBM_PEAK_GBS = 8000.0            # MI355X HBM3E peak, vendor figure

# HBM bytes per launch of the score kernels, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of
# this script (summary and commands: profiles/hbm_traffic_bench_cfg3.md; FETCH_SIZE scaled x2.0 and
# WRITE_SIZE x1.0 by what the same counters read for a plain 256 MiB copy).  Counters cannot be read
# from inside the timed run, so the figure is carried here; None for workloads not profiled.
MEASURED_TRAFFIC_BYTES = {
    ("cfg3_llama3_8b_gqa_s16384", "colsum_kernel"): (186578.0 * 2.0 + 4327.1) * 1024.0,
    ("cfg3_llama3_8b_gqa_s16384", "lse_kernel"): (115738.4 * 2.0 + 2048.0) * 1024.0,
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=32)
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--config", type=int, default=3, help="workload id 1..5 (default: the S=16384 GQA layer)")
    ap.add_argument("--layers", type=int, default=0, help="resident layers (0: the workload's own count, capped at 32)")
    ap.add_argument("--window", type=int, default=0,
                    help="observation window W: only the last W queries score the tokens (SnapKV-style scoring)")
    ap.add_argument("--pool", type=int, default=0, help="max-pool the scores with this odd kernel before selection")
    ap.add_argument("--lse-supplied", action="store_true",
                    help="informational: the row normalisers come from the attention kernel (computed before the "
                         "timed region), stage 1 is then one sweep; not the headline configuration")
    ap.add_argument("--unit", type=int, default=0,
                    help="chunk- / page-level selection on units of this many tokens (0: token level)")
    ap.add_argument("--decode", action="store_true",
                    help="time the decoding-time score append on caches of --cache-len tokens instead of the "
                         "per-layer compression step")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step per resident layer (or cache, with --decode) in a HIP graph and time "
                         "replays; stage times still come from the eager pass")
    ap.add_argument("--cache-len", type=int, default=0, help="--decode: valid tokens per cache (0: the workload's budget)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--overlap", action="store_true",
                    help="also time the steps on two streams (a layer's selection beside the next layer's scores) "
                         "and report that as ms_per_step; stage times stay those of the one-stream run")
    ap.add_argument("--no-mfma-ceiling", action="store_true",
                    help="skip the MFMA-only calibration launch that follows the timed region")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (reference for HBM byte counters)")
    return ap.parse_args()


def mfma_ceiling_tflops(torch, dev, q_sample):
    """What the matrix pipe sustains on v_mfma_f32_32x32x16_bf16 alone (no LDS traffic, no vector ALU
    work) with operands drawn from the workload's own Q values: the measured counterpart of the
    datasheet peak.  The kernel lives in the separate calibration library."""
    import ctypes
    from paper_2503_00022_amd import build as b
    L = ctypes.CDLL(b.BENCH_LIB_PATH)
    L.kvcrush_bench_mfma_ceiling.restype = ctypes.c_double
    L.kvcrush_bench_mfma_ceiling.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p,
                                             ctypes.c_void_p]
    L.kvcrush_bench_mfma_operand_bytes.restype = ctypes.c_size_t
    need = L.kvcrush_bench_mfma_operand_bytes()
    ops = q_sample.reshape(-1).view(torch.uint8)[:need].contiguous()
    assert ops.numel() == need, "sample too small for the calibration kernel's operands"
    grid, iters = 512, 4096                                  # two workgroups per compute unit, about 1 ms
    out = torch.empty(grid * 256, dtype=torch.float32, device=dev)
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    best = 0.0
    for rep in range(6):                                     # the first launches also settle the clock
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        flop = L.kvcrush_bench_mfma_ceiling(ops.data_ptr(), iters, grid, out.data_ptr(), st)
        e1.record()
        torch.cuda.synchronize()
        if flop <= 0.0:
            return None
        if rep >= 2:
            best = max(best, flop / (e0.elapsed_time(e1) * 1e-3) / 1e12)
    return best


def cpu_baseline(w, q0, k0, v0, sc_gpu_layer0, layer, row_begin=0, pool=0, unit=0):
    """The oracle as it stands, single-threaded, on a bounded sample: every query
    row of the first few query heads of layer 0 (heads are added until about 12 s
    of CPU work are spent), plus the full selection and gather of that layer.
    Extrapolated to a whole layer."""
    import oracle
    import torch
    from paper_2503_00022_amd import inputs

    G = w.Hq // w.Hkv
    t_heads, n_heads = 0.0, 0
    while n_heads < min(w.Hq, 8) and (n_heads == 0 or t_heads < 12.0):
        q_h = q0[0, n_heads].cpu()
        k_h = k0[0, n_heads // G].cpu()
        t0 = time.perf_counter()
        oracle.head_colsums(q_h, k_h, row_begin, w.S)
        t_heads += time.perf_counter() - t0
        n_heads += 1
    t_head = t_heads / n_heads
    sc = sc_gpu_layer0.cpu()
    t0 = time.perf_counter()
    if pool:
        sc = oracle.maxpool(sc, pool)
    if unit > 1:
        idx, _, _ = oracle.select_units(sc, unit, w.budget, w.n_important, 0, w.anchor, inputs.anchor_seed(layer))
    else:
        idx, _, _ = oracle.select(sc, w.budget, w.n_important, 0, w.anchor, inputs.anchor_seed(layer))
    t_sel = time.perf_counter() - t0
    kc, vc = k0.cpu(), v0.cpu()
    t0 = time.perf_counter()
    oracle.compact(kc, vc, idx)
    t_cmp = time.perf_counter() - t0
    t_layer = t_head * w.Hq * w.B + t_sel + t_cmp
    return {
        "value": w.B * w.S / t_layer, "unit": "tokens/s", "cores": 1, "kind": "oracle",
        "sample": (f"layer 0: query rows {row_begin}..{w.S - 1} of {n_heads} of {w.B * w.Hq} (sequence, query head) pairs "
                   f"timed ({t_heads:.2f} s) and scaled by {w.B * w.Hq}/{n_heads}; selection ({t_sel:.3f} s) and gather "
                   f"({t_cmp:.3f} s) timed in full"),
        "seconds_per_layer_extrapolated": t_layer,
    }


def run_decode(args, torch, kv, inputs, dev):
    """One step = one decoded token per sequence of the batch: kvcrush_scores_append on a cache of
    --cache-len tokens.  Several caches are walked in turn so that the last-level cache cannot hold K."""
    w = inputs.CONFIGS[args.config]
    S = args.cache_len or w.budget
    cap = S + 256
    Hs = w.Hs
    esz = 2 if w.dtype == "bf16" else 4
    k_bytes = w.B * w.Hkv * S * w.D * esz
    n_caches = max(2, min(32, int(1.5e9 // max(k_bytes, 1))))
    g = torch.Generator(device=dev).manual_seed(inputs.BASE_SEED)
    caches = []
    for _ in range(n_caches):
        kc = torch.randn(w.B, w.Hkv, cap, w.D, generator=g, device=dev).to(w.torch_dtype)
        qn = torch.randn(w.B, w.Hq, w.D, generator=g, device=dev).to(w.torch_dtype)
        sc = torch.rand(w.B, Hs, cap, generator=g, device=dev)
        caches.append((qn, kc, sc))
    shape = kv.Shape(w.B, w.Hq, w.Hkv, S, w.D, kv.BF16 if w.dtype == "bf16" else kv.F32, int(w.reduce_groups), 0)
    ws = torch.empty(max(kv.kvcrush_scores_append_workspace(shape, cap), 16), dtype=torch.uint8, device=dev)

    def step(i):
        qn, kc, sc = caches[i % n_caches]
        kv.kvcrush_scores_append(qn, kc, sc, S, w.reduce_groups, workspace=ws)

    for i in range(max(args.warmup, n_caches if args.graph else 0)):
        step(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    if args.graph:
        graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for i in range(n_caches):
                    step(i)
        torch.cuda.synchronize()
        replays = max(1, args.steps // n_caches)
        args.steps = replays * n_caches
        t0 = time.perf_counter()
        e0.record()
        for _ in range(replays):
            graph.replay()
        e1.record()
    else:
        t0 = time.perf_counter()
        e0.record()
        for i in range(args.steps):
            step(args.warmup + i)
        e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    gpu_ms = e0.elapsed_time(e1) / args.steps
    ms = wall * 1e3 / args.steps
    out = {
        "metric": "decode_score_append_tokens_per_sec", "value": w.B / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}_decode_cache{S}", "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "cache_len": S,
                   "capacity": cap, "D": w.D, "reduce_groups": w.reduce_groups, "resident_caches": n_caches,
                   "hip_graph": args.graph},
        "roofline": {"bound": "hbm", "kernel": "append_logits_kernel + append_update_kernel",
                     "achieved": k_bytes / (gpu_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": k_bytes / (gpu_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "traffic": None,
                     "bytes_per_step": k_bytes, "avg_step_gpu_ms": gpu_ms},
    }
    print(json.dumps(out), flush=True)


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (the path has no cross-GPU step); "
              "run it with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2503_00022_amd import binding as kv
    from paper_2503_00022_amd import inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    from paper_2503_00022_amd import build as _build
    _build.ensure_built()   # compiles only when no library is there
    kv.load()
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    if args.decode:
        return run_decode(args, torch, kv, inputs, dev)
    w = inputs.CONFIGS[args.config]
    n_layers = args.layers or min(w.layers, 32)
    # a single-layer workload still rotates over a few copies so that repeats miss the cache
    if w.layers == 1 and not args.layers:
        n_layers = 4
    G = w.Hq // w.Hkv
    Hs = w.Hs

    layers = []
    for L in range(n_layers):
        q, k, v = inputs.make_qkv(w, inputs.layer_seed(args.config, L), device=dev)
        ent = {"q": q, "k": k, "v": v}
        if w.paged:
            bt = inputs.make_block_table(w, inputs.layer_seed(args.config, L))
            ent["bt"] = bt.to(dev)
            ent["kp"] = inputs.to_paged(k, bt, w.block_size)
            ent["vp"] = inputs.to_paged(v, bt, w.block_size)
        layers.append(ent)
    torch.cuda.synchronize()

    W = args.window if 0 < args.window < w.S else 0
    q_first = w.S - W if W else 0
    pooled = torch.empty(w.B, Hs, w.S, dtype=torch.float32, device=dev) if args.pool else None
    lse = torch.empty(w.B, w.Hq, w.S, dtype=torch.float32, device=dev)
    shape = kv.make_shape(layers[0]["q"], layers[0]["k"], w.reduce_groups, W)
    lse_ws = torch.empty(max(kv.kvcrush_row_lse_workspace(shape), 16), dtype=torch.uint8, device=dev)
    sc_ws = torch.empty(max(kv.kvcrush_scores_workspace(shape), 16), dtype=torch.uint8, device=dev)
    scores = torch.empty(w.B, Hs, w.S, dtype=torch.float32, device=dev)
    idx = torch.empty(w.B, w.budget, dtype=torch.int32, device=dev)
    sel_ws = torch.empty(kv.kvcrush_select_workspace(
        kv.make_select_args(w.B, Hs, w.S, w.budget, w.n_important, unit=args.unit)), dtype=torch.uint8, device=dev)
    k_out = torch.empty(w.B, w.Hkv, w.budget, w.D, dtype=w.torch_dtype, device=dev)
    v_out = torch.empty_like(k_out)

    if args.lse_supplied:
        for ent in layers:
            ent["lse"] = kv.kvcrush_row_lse(ent["q"], ent["k"], window=W, workspace=lse_ws)
        torch.cuda.synchronize()

    def step(i, ev=None):
        L = i % n_layers
        ent = layers[L]
        if ev:
            ev[0].record()
        if not args.lse_supplied:
            kv.kvcrush_row_lse(ent["q"], ent["k"], lse_out=lse, window=W, workspace=lse_ws)
        if ev:
            ev[1].record()
        kv.kvcrush_scores(ent["q"], ent["k"], w.reduce_groups, lse=ent["lse"] if args.lse_supplied else lse,
                          scores=scores, window=W, workspace=sc_ws)
        if ev:
            ev[2].record()
        if pooled is not None:
            kv.kvcrush_pool_scores(scores, args.pool, out=pooled)
        kv.kvcrush_select(scores if pooled is None else pooled, w.budget, w.n_important, 0, w.anchor,
                          inputs.anchor_seed(L), want_kind=False, idx=idx, workspace=sel_ws, unit=args.unit)
        if ev:
            ev[3].record()
        if w.paged:
            kv.kvcrush_compact(ent["kp"], ent["vp"], idx, block_table=ent["bt"], block_size=w.block_size,
                               dense_shape=(w.B, w.Hkv, w.S, w.D), k_out=k_out, v_out=v_out, validate=False)
        else:
            kv.kvcrush_compact(ent["k"], ent["v"], idx, k_out=k_out, v_out=v_out, validate=False)
        if ev:
            ev[4].record()

    copy_gbs = None
    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        dst.copy_(src)       # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        c0.record()
        for _ in range(10):
            dst.copy_(src)
        c1.record()
        torch.cuda.synchronize()
        copy_gbs = 10 * 2.0 * (256 << 20) / (c0.elapsed_time(c1) * 1e-3) / 1e9   # read + write
        del src, dst

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i, evs[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    ms_per_step = wall * 1e3 / args.steps
    eager_ms_per_step = ms_per_step
    if args.graph:
        # the same steps, one per resident layer, captured once and replayed: launch cost off the host
        graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for i in range(n_layers):
                    step(i)
        torch.cuda.synchronize()
        replays = max(1, args.steps // n_layers)
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(replays):
            graph.replay()
        torch.cuda.synchronize()
        ms_per_step = (time.perf_counter() - t0) * 1e3 / (replays * n_layers)
    if args.overlap:
        # the same steps on two streams: layer L's selection and gather (a few compute units, bound by
        # latency) run beside layer L+1's score kernels; the scores are double-buffered between them
        s_sel = torch.cuda.Stream()
        sc2 = [scores, torch.empty_like(scores)]
        ready = [torch.cuda.Event() for _ in range(2)]
        done = [torch.cuda.Event() for _ in range(2)]
        main = torch.cuda.current_stream()

        def step2(i):
            L, j = i % n_layers, i % 2
            ent = layers[L]
            if i >= 2:
                main.wait_event(done[j])          # the selection two steps back has read this buffer
            if not args.lse_supplied:
                kv.kvcrush_row_lse(ent["q"], ent["k"], lse_out=lse, window=W, workspace=lse_ws)
            kv.kvcrush_scores(ent["q"], ent["k"], w.reduce_groups, lse=ent["lse"] if args.lse_supplied else lse,
                              scores=sc2[j], window=W, workspace=sc_ws)
            ready[j].record(main)
            with torch.cuda.stream(s_sel):
                s_sel.wait_event(ready[j])
                src = sc2[j]
                if pooled is not None:
                    src = kv.kvcrush_pool_scores(sc2[j], args.pool, out=pooled)
                kv.kvcrush_select(src, w.budget, w.n_important, 0, w.anchor, inputs.anchor_seed(L), want_kind=False,
                                  idx=idx, workspace=sel_ws, unit=args.unit)
                if w.paged:
                    kv.kvcrush_compact(ent["kp"], ent["vp"], idx, block_table=ent["bt"], block_size=w.block_size,
                                       dense_shape=(w.B, w.Hkv, w.S, w.D), k_out=k_out, v_out=v_out, validate=False)
                else:
                    kv.kvcrush_compact(ent["k"], ent["v"], idx, k_out=k_out, v_out=v_out, validate=False)
                done[j].record(s_sel)

        for i in range(max(args.warmup, 2)):
            step2(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step2(i)
        torch.cuda.synchronize()
        ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
        # the last overlapped step against the same layer run on one stream
        idx_two = idx.clone()
        step(args.steps - 1)
        torch.cuda.synchronize()
        overlap_ok = bool(torch.equal(idx_two, idx))
    stage = [sum(e[j].elapsed_time(e[j + 1]) for e in evs) / args.steps for j in range(4)]  # ms
    t_lse, t_col, t_sel, t_cmp = stage
    med = [sorted(e[j].elapsed_time(e[j + 1]) for e in evs)[len(evs) // 2] for j in range(4)]
    tokens = w.B * w.S

    # algorithmic work (what the method must compute / move, not what a kernel happens to do)
    pairs = w.S * (w.S + 1) // 2 - q_first * (q_first + 1) // 2   # causal (query, key) pairs per head
    flop_pass = 2.0 * w.D * pairs * w.Hq * w.B                    # one sweep of Q K^T
    esz = 2 if w.dtype == "bf16" else 4
    bytes_sel = 4.0 * Hs * w.S * w.B + 4.0 * w.budget * w.B
    bytes_cmp = 2.0 * 2.0 * w.B * w.Hkv * w.budget * w.D * esz + 4.0 * w.budget * w.B
    dom_name, dom_ms = ("colsum_kernel", t_col) if t_col >= t_lse else ("lse_kernel", t_lse)
    n_sweeps = 1 if args.lse_supplied else 2
    achieved = flop_pass / (dom_ms * 1e-3) / 1e12
    peak = MFMA_BF16_PEAK_TFLOPS if w.dtype == "bf16" else 157.3
    traffic = MEASURED_TRAFFIC_BYTES.get((w.name, dom_name)) if not W else None
    roofline = {
        "bound": "mfma", "kernel": dom_name, "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
        "frac": achieved / peak, "traffic": traffic,
        "flop_per_launch": flop_pass, "avg_launch_ms": dom_ms,
    }
    stages = {
        "lse_ms": t_lse, "colsum_ms": t_col, "select_ms": t_sel, "compact_ms": t_cmp,
        "scores_tflops": n_sweeps * flop_pass / ((t_lse + t_col) * 1e-3) / 1e12,
        "scores_frac_of_mfma_peak": n_sweeps * flop_pass / ((t_lse + t_col) * 1e-3) / 1e12 / peak,
        "select_compact_gbs": (bytes_sel + bytes_cmp) / ((t_sel + t_cmp) * 1e-3) / 1e9,
        "select_compact_frac_of_hbm_peak": (bytes_sel + bytes_cmp) / ((t_sel + t_cmp) * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "compact_gbs": bytes_cmp / (t_cmp * 1e-3) / 1e9,
        "median_ms": {"lse": med[0], "colsum": med[1], "select": med[2], "compact": med[3]},
    }

    # cheap sanity check of the last step's scores: every row totals (group size) x S
    tot = scores.double().sum(-1)
    want = float((G if w.reduce_groups else 1) * (w.S - q_first))
    ok = bool(torch.allclose(tot, torch.full_like(tot, want), rtol=1e-4))

    out = {
        "metric": "kv_compressed_tokens_per_sec_per_layer", "value": tokens / (ms_per_step * 1e-3),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "S": w.S, "D": w.D,
                   "budget": w.budget, "n_important": w.n_important, "n_representative": w.n_rep,
                   "anchor": w.anchor, "reduce_groups": w.reduce_groups, "paged": w.paged,
                   "resident_layers": n_layers, "obs_window": W, "pool_kernel": args.pool, "unit": args.unit, "lse_supplied": args.lse_supplied,
                   "launch": "hip_graph" if args.graph else ("eager, two streams" if args.overlap else "eager")},
        "roofline": roofline, "stages": stages, "row_sum_check": ok,
    }
    if args.graph or args.overlap:
        out["eager_ms_per_step"] = eager_ms_per_step   # one stream, one launch after the other
    if args.overlap:
        out["overlap_check"] = overlap_ok
    if w.dtype == "bf16" and not args.no_mfma_ceiling:
        # measured counterpart of the datasheet peak, taken after the timed region
        ceil = mfma_ceiling_tflops(torch, dev, layers[0]["q"])
        if ceil:
            roofline["measured_mfma_only_tflops"] = ceil
            roofline["frac_of_measured"] = achieved / ceil
    if copy_gbs is not None:
        out["plain_copy_gbs"] = copy_gbs   # the runtime's device-to-device copy of 256 MiB, read + write
    if not args.no_cpu_baseline:
        # layer 0 again, so that its scores are the ones handed to the oracle's selection
        step(0)
        torch.cuda.synchronize()
        out["cpu_baseline"] = cpu_baseline(w, layers[0]["q"], layers[0]["k"], layers[0]["v"], scores, 0,
                                           q_first, args.pool, args.unit)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
