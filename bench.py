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
    ("cfg3_llama3_8b_gqa_s16384", "colsum_kernel"): (197737.1 * 2.0 + 4320.0) * 1024.0,
    ("cfg3_llama3_8b_gqa_s16384", "lse_kernel"): (118440.3 * 2.0 + 2048.0) * 1024.0,
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
                    help="(kept for the profiling commands: the 256 MiB device copies that serve as the reference "
                         "for the HBM byte counters are always run now)")
    ap.add_argument("--per-head-bits", action="store_true",
                    help="one score row (one bit of the vector) per query head instead of per KV group")
    ap.add_argument("--quick", action="store_true",
                    help="only the main workload's eager run: no HIP-graph figure, no short runs of the other workloads")
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


def mix_ceiling_tflops(torch, dev, q_sample):
    """What the chip sustains on the score kernels' instruction mix alone: per 64 x 32 block 16 MFMAs
    and, for each of the previous block's 32 accumulator values, multiply-add, exp2 and add, interleaved
    as in the kernels; no memory traffic (csrc/bench/mix_ceiling.hip).  Matrix FLOP/s, like the kernels'."""
    import ctypes
    from paper_2503_00022_amd import build as b
    L = ctypes.CDLL(b.BENCH_LIB_PATH)
    L.kvcrush_bench_mix_ceiling.restype = ctypes.c_double
    L.kvcrush_bench_mix_ceiling.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p,
                                            ctypes.c_void_p]
    L.kvcrush_bench_mix_operand_bytes.restype = ctypes.c_size_t
    need = L.kvcrush_bench_mix_operand_bytes()
    ops = q_sample.reshape(-1).view(torch.uint8)[:need].contiguous()
    assert ops.numel() == need, "sample too small for the calibration kernel's operands"
    grid, iters = 512, 1024                                  # two workgroups per compute unit, about 1 ms
    out = torch.empty(grid * 256, dtype=torch.float32, device=dev)
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    best = 0.0
    for rep in range(6):                                     # the first launches also settle the clock
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        flop = L.kvcrush_bench_mix_ceiling(ops.data_ptr(), iters, grid, out.data_ptr(), st)
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


def copy_ceiling_gbs(torch, dev):
    """Measured counterpart of the HBM datasheet peak: the runtime's own device-to-device copy of
    256 MiB (read + write), 10 copies timed."""
    src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(10):
        dst.copy_(src)
    c1.record()
    torch.cuda.synchronize()
    return 10 * 2.0 * (256 << 20) / (c0.elapsed_time(c1) * 1e-3) / 1e9


class Run:
    """One workload resident in HBM with its buffers; step(i) enqueues one layer's compression."""

    def __init__(self, torch, kv, inputs, dev, cfg_id, w, n_layers, args):
        self.torch, self.kv, self.inputs, self.w, self.args, self.n_layers = torch, kv, inputs, w, args, n_layers
        Hs = w.Hs
        self.layers = []
        for L in range(n_layers):
            q, k, v = inputs.make_qkv(w, inputs.layer_seed(cfg_id, L), device=dev)
            ent = {"q": q, "k": k, "v": v}
            if w.paged:
                bt = inputs.make_block_table(w, inputs.layer_seed(cfg_id, L))
                ent["bt"] = bt.to(dev)
                ent["kp"] = inputs.to_paged(k, bt, w.block_size)
                ent["vp"] = inputs.to_paged(v, bt, w.block_size)
            self.layers.append(ent)
        torch.cuda.synchronize()
        self.W = args.window if 0 < args.window < w.S else 0
        self.q_first = w.S - self.W if self.W else 0
        self.pooled = torch.empty(w.B, Hs, w.S, dtype=torch.float32, device=dev) if args.pool else None
        self.lse = torch.empty(w.B, w.Hq, w.S, dtype=torch.float32, device=dev)
        shape = kv.make_shape(self.layers[0]["q"], self.layers[0]["k"], w.reduce_groups, self.W)
        self.lse_ws = torch.empty(max(kv.kvcrush_row_lse_workspace(shape), 16), dtype=torch.uint8, device=dev)
        self.sc_ws = torch.empty(max(kv.kvcrush_scores_workspace(shape), 16), dtype=torch.uint8, device=dev)
        self.scores = torch.empty(w.B, Hs, w.S, dtype=torch.float32, device=dev)
        self.idx = torch.empty(w.B, w.budget, dtype=torch.int32, device=dev)
        self.sel_ws = torch.empty(kv.kvcrush_select_workspace(
            kv.make_select_args(w.B, Hs, w.S, w.budget, w.n_important, unit=args.unit)), dtype=torch.uint8, device=dev)
        self.k_out = torch.empty(w.B, w.Hkv, w.budget, w.D, dtype=w.torch_dtype, device=dev)
        self.v_out = torch.empty_like(self.k_out)
        if args.lse_supplied:
            for ent in self.layers:
                ent["lse"] = kv.kvcrush_row_lse(ent["q"], ent["k"], window=self.W, workspace=self.lse_ws)
            torch.cuda.synchronize()

    def select_and_gather(self, L, scores, ev=None):
        kv, w, args, ent = self.kv, self.w, self.args, self.layers[L]
        src = scores
        if self.pooled is not None:
            src = kv.kvcrush_pool_scores(scores, args.pool, out=self.pooled)
        kv.kvcrush_select(src, w.budget, w.n_important, 0, w.anchor, self.inputs.anchor_seed(L), want_kind=False,
                          idx=self.idx, workspace=self.sel_ws, unit=args.unit)
        if ev:
            ev.record()
        if w.paged:
            kv.kvcrush_compact(ent["kp"], ent["vp"], self.idx, block_table=ent["bt"], block_size=w.block_size,
                               dense_shape=(w.B, w.Hkv, w.S, w.D), k_out=self.k_out, v_out=self.v_out, validate=False)
        else:
            kv.kvcrush_compact(ent["k"], ent["v"], self.idx, k_out=self.k_out, v_out=self.v_out, validate=False)

    def timed(self, steps, warmup):
        """`warmup` untimed steps, then `steps` timed ones on one stream with HIP events between the
        stages.  Returns wall ms per step and the per-stage event times (lists of ms)."""
        torch = self.torch
        for i in range(warmup):
            self.step_with_events(i, None)
        torch.cuda.synchronize()
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(steps)]
        t0 = time.perf_counter()
        for i in range(steps):
            self.step_with_events(warmup + i, evs[i])
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        return wall * 1e3 / steps, [[e[j].elapsed_time(e[j + 1]) for e in evs] for j in range(4)]

    def step_with_events(self, i, ev):
        kv, w, args = self.kv, self.w, self.args
        L = i % self.n_layers
        ent = self.layers[L]
        if ev:
            ev[0].record()
        if not args.lse_supplied:
            kv.kvcrush_row_lse(ent["q"], ent["k"], lse_out=self.lse, window=self.W, workspace=self.lse_ws)
        if ev:
            ev[1].record()
        kv.kvcrush_scores(ent["q"], ent["k"], w.reduce_groups, lse=ent["lse"] if args.lse_supplied else self.lse,
                          scores=self.scores, window=self.W, workspace=self.sc_ws)
        if ev:
            ev[2].record()
        self.select_and_gather(L, self.scores, ev[3] if ev else None)
        if ev:
            ev[4].record()

    def graph_ms_per_step(self, steps):
        """The same steps, one per resident layer, captured once in a HIP graph and replayed."""
        torch = self.torch
        graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for i in range(self.n_layers):
                    self.step_with_events(i, None)
        torch.cuda.synchronize()
        replays = max(1, steps // self.n_layers)
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(replays):
            graph.replay()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / (replays * self.n_layers)

    def overlap_ms_per_step(self, steps, warmup):
        """The same steps on two streams: layer L's selection and gather (a few compute units, bound by
        latency) run beside layer L+1's score kernels; the scores are double-buffered between them."""
        torch, kv, w, args = self.torch, self.kv, self.w, self.args
        s_sel = torch.cuda.Stream()
        sc2 = [self.scores, torch.empty_like(self.scores)]
        ready = [torch.cuda.Event() for _ in range(2)]
        done = [torch.cuda.Event() for _ in range(2)]
        main = torch.cuda.current_stream()

        def step2(i):
            L, j = i % self.n_layers, i % 2
            ent = self.layers[L]
            if i >= 2:
                main.wait_event(done[j])          # the selection two steps back has read this buffer
            if not args.lse_supplied:
                kv.kvcrush_row_lse(ent["q"], ent["k"], lse_out=self.lse, window=self.W, workspace=self.lse_ws)
            kv.kvcrush_scores(ent["q"], ent["k"], w.reduce_groups, lse=ent["lse"] if args.lse_supplied else self.lse,
                              scores=sc2[j], window=self.W, workspace=self.sc_ws)
            ready[j].record(main)
            with torch.cuda.stream(s_sel):
                s_sel.wait_event(ready[j])
                self.select_and_gather(L, sc2[j])
                done[j].record(s_sel)

        for i in range(max(warmup, 2)):
            step2(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            step2(i)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        idx_two = self.idx.clone()                # the last overlapped step against the same layer on one stream
        self.step_with_events(steps - 1, None)
        torch.cuda.synchronize()
        return ms, bool(torch.equal(idx_two, self.idx))

    def figures(self, ms_per_step, stage_ms):
        """Per-stage rates from the algorithmic work (what the method must compute or move, not what a
        kernel happens to do) and the event times."""
        w, args = self.w, self.args
        t_lse, t_col, t_sel, t_cmp = [sum(x) / len(x) for x in stage_ms]
        med = [sorted(x)[len(x) // 2] for x in stage_ms]
        q_first = self.q_first
        pairs = w.S * (w.S + 1) // 2 - q_first * (q_first + 1) // 2   # causal (query, key) pairs per head
        flop_pass = 2.0 * w.D * pairs * w.Hq * w.B                    # one sweep of Q K^T
        esz = 2 if w.dtype in ("bf16", "f16") else 4
        bytes_sel = 4.0 * w.Hs * w.S * w.B + 4.0 * w.budget * w.B
        bytes_cmp = 2.0 * 2.0 * w.B * w.Hkv * w.budget * w.D * esz + 4.0 * w.budget * w.B
        n_sweeps = 1 if args.lse_supplied else 2
        peak = MFMA_BF16_PEAK_TFLOPS if w.dtype == "bf16" else 157.3
        t_scores = (t_lse + t_col) if not args.lse_supplied else t_col
        stages = {
            "lse_ms": t_lse, "colsum_ms": t_col, "select_ms": t_sel, "compact_ms": t_cmp,
            "scores_tflops": n_sweeps * flop_pass / (t_scores * 1e-3) / 1e12,
            "scores_frac_of_mfma_peak": n_sweeps * flop_pass / (t_scores * 1e-3) / 1e12 / peak,
            "select_compact_gbs": (bytes_sel + bytes_cmp) / ((t_sel + t_cmp) * 1e-3) / 1e9,
            "select_compact_frac_of_hbm_peak": (bytes_sel + bytes_cmp) / ((t_sel + t_cmp) * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "compact_gbs": bytes_cmp / (t_cmp * 1e-3) / 1e9,
            "median_ms": {"lse": med[0], "colsum": med[1], "select": med[2], "compact": med[3]},
        }
        return stages, flop_pass, peak

    def row_sum_check(self):
        """Cheap sanity check of the last step's scores: every row totals (group size) x query rows."""
        torch, w = self.torch, self.w
        tot = self.scores.double().sum(-1)
        want = float((w.Hq // w.Hkv if w.reduce_groups else 1) * (w.S - self.q_first))
        return bool(torch.allclose(tot, torch.full_like(tot, want), rtol=1e-4))

    def config(self, launch):
        w, args = self.w, self.args
        return {"workload": w.name, "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "S": w.S, "D": w.D,
                "budget": w.budget, "n_important": w.n_important, "n_representative": w.n_rep,
                "anchor": w.anchor, "reduce_groups": w.reduce_groups, "paged": w.paged,
                "resident_layers": self.n_layers, "obs_window": self.W, "pool_kernel": args.pool, "unit": args.unit,
                "lse_supplied": args.lse_supplied, "launch": launch}


def other_configs(torch, kv, inputs, dev, args, headline_id):
    """Short timed runs of the other workloads (a few steps each, two or three resident layers), so that
    one driver run shows every configuration; the headline figure stays the main workload's."""
    import dataclasses
    rows = []
    todo = [(c, inputs.CONFIGS[c], f"cfg{c}") for c in (1, 2, 3, 4, 5) if c != headline_id]
    # one bit per query head at full GQA size (Sec. 4.3.3 counts 32 bits per token for a Llama-3-8B layer)
    todo.append((3, dataclasses.replace(inputs.CONFIGS[3], name="cfg3_per_query_head_bits", reduce_groups=False),
                 "cfg3 with one score row per query head"))
    for cfg_id, w, label in todo:
        n_layers = 3 if w.B * w.S <= 16384 else 2
        run = Run(torch, kv, inputs, dev, cfg_id, w, n_layers, args)
        steps = 6
        ms, stage_ms = run.timed(steps, 2)
        stages, _, _ = run.figures(ms, stage_ms)
        rows.append({"workload": w.name, "note": label, "steps": steps, "resident_layers": n_layers, "dtype": w.dtype,
                     "ms_per_step": ms, "tokens_per_s": w.B * w.S / (ms * 1e-3),
                     "scores_frac_of_mfma_peak": stages["scores_frac_of_mfma_peak"], "lse_ms": stages["lse_ms"],
                     "colsum_ms": stages["colsum_ms"], "select_ms": stages["select_ms"],
                     "compact_ms": stages["compact_ms"], "compact_gbs": stages["compact_gbs"],
                     "row_sum_check": run.row_sum_check()})
        del run
        torch.cuda.empty_cache()
    return rows


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
    if args.per_head_bits:
        import dataclasses
        w = dataclasses.replace(w, name=w.name + "_per_query_head_bits", reduce_groups=False)
    n_layers = args.layers or min(w.layers, 32)
    # a single-layer workload still rotates over a few copies so that repeats miss the cache
    if w.layers == 1 and not args.layers:
        n_layers = 4

    copy_gbs = copy_ceiling_gbs(torch, dev)
    run = Run(torch, kv, inputs, dev, args.config, w, n_layers, args)
    ms_per_step, stage_ms = run.timed(args.steps, args.warmup)      # the headline: eager, one stream
    eager_ms_per_step = ms_per_step
    launch = "eager"
    graph_ms = None
    if args.graph or not args.quick:
        graph_ms = run.graph_ms_per_step(args.steps)
    if args.graph:
        ms_per_step, launch = graph_ms, "hip_graph"
    overlap_ms = overlap_ok = None
    if args.overlap or not args.quick:
        overlap_ms, overlap_ok = run.overlap_ms_per_step(args.steps, args.warmup)
    if args.overlap:
        ms_per_step, launch = overlap_ms, "eager, two streams"
    stages, flop_pass, peak = run.figures(ms_per_step, stage_ms)
    t_lse, t_col = stages["lse_ms"], stages["colsum_ms"]
    # (the events bracket the library call: pass B's time includes its 4 us partial-sum reduction)
    dom_name, dom_ms = ("colsum_kernel", t_col) if t_col >= t_lse else ("lse_kernel", t_lse)
    achieved = flop_pass / (dom_ms * 1e-3) / 1e12
    traffic = MEASURED_TRAFFIC_BYTES.get((w.name, dom_name)) if not run.W else None
    roofline = {
        "bound": "mfma", "kernel": dom_name, "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
        "frac": achieved / peak, "traffic": traffic,
        "flop_per_launch": flop_pass, "avg_launch_ms": dom_ms,
    }
    stages["select_compact_frac_of_measured_copy"] = stages["select_compact_gbs"] / copy_gbs
    stages["compact_frac_of_hbm_peak"] = stages["compact_gbs"] / HBM_PEAK_GBS
    stages["compact_frac_of_measured_copy"] = stages["compact_gbs"] / copy_gbs

    tokens = w.B * w.S
    out = {
        "metric": "kv_compressed_tokens_per_sec_per_layer", "value": tokens / (ms_per_step * 1e-3),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic", "config": run.config(launch),
        "roofline": roofline, "stages": stages, "row_sum_check": run.row_sum_check(),
        "plain_copy_gbs": copy_gbs,   # the runtime's device-to-device copy of 256 MiB, read + write
    }
    if graph_ms is not None:
        out["graph_ms_per_step"] = graph_ms          # the same steps replayed from a HIP graph (informational)
    if args.graph or args.overlap:
        out["eager_ms_per_step"] = eager_ms_per_step   # one stream, one launch after the other
    if overlap_ms is not None:
        # layer L's selection and gather on a second stream beside layer L + 1's score kernels (informational)
        out["overlap_ms_per_step"] = overlap_ms
        out["overlap_check"] = overlap_ok            # the overlapped run's last index list equals the one-stream one
    if w.dtype == "bf16" and not args.no_mfma_ceiling:
        # measured counterparts of the datasheet peak, taken after the timed region
        ceil = mfma_ceiling_tflops(torch, dev, run.layers[0]["q"])
        if ceil:
            roofline["measured_mfma_only_tflops"] = ceil
            roofline["frac_of_measured"] = achieved / ceil
        mix = mix_ceiling_tflops(torch, dev, run.layers[0]["q"])
        if mix:
            roofline["measured_mix_tflops"] = mix          # 16 MFMAs + 32 x (fma, exp2, add) per block, nothing else
            roofline["frac_of_measured_mix"] = achieved / mix
    if not args.no_cpu_baseline:
        # layer 0 again, so that its scores are the ones handed to the oracle's selection
        run.step_with_events(0, None)
        torch.cuda.synchronize()
        out["cpu_baseline"] = cpu_baseline(w, run.layers[0]["q"], run.layers[0]["k"], run.layers[0]["v"],
                                           run.scores, 0, run.q_first, args.pool, args.unit)
    if not args.quick and not (args.window or args.pool or args.unit or args.lse_supplied):
        del run
        torch.cuda.empty_cache()
        out["configs"] = other_configs(torch, kv, inputs, dev, args, None if args.per_head_bits else args.config)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
