"""ctypes access to the CPU oracle (oracle/kvcrush_oracle.cpp).

TEST INFRASTRUCTURE ONLY.  Only tests, the smoke check and the benchmark's
CPU-baseline leg may import this package; the GPU library and its Python
binding never do.  Tensors are torch CPU tensors (contiguous); nothing here
touches a GPU.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import torch

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "kvcrush_oracle.cpp")
_LIB = os.path.join(_DIR, "libkvcrush_oracle.so")
# The mutation tests (tests/test_oracle_mutations.py) point this at a copy of the oracle with a
# planted mistake to show that the pins notice it; nothing else sets it.
_LIB_OVERRIDE = os.environ.get("KVCRUSH_ORACLE_LIB_FOR_MUTATION_TEST")
CXXFLAGS = ["-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC"]

F32, BF16, F16 = 0, 1, 2
ANCHOR_RANDOM, ANCHOR_MEAN, ANCHOR_ALTERNATING, ANCHOR_EXPLICIT = 0, 1, 2, 3
ANCHORS = {"random": 0, "mean": 1, "alternating": 2, "explicit": 3}


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (single translation unit, no dependencies)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.run(["g++", *CXXFLAGS, "-o", tmp, _SRC], check=True)
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(_LIB_OVERRIDE or build())
        vp, i32, u64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64
        f64 = ctypes.c_double
        L.kvcrush_oracle_head_colsums.argtypes = [i32, i32, i32, vp, vp, i32, i32, f64, vp, vp]
        L.kvcrush_oracle_scores.argtypes = [i32] * 8 + [f64] + [vp] * 4
        L.kvcrush_oracle_maxpool.argtypes = [i32, i32, i32, vp, vp]
        L.kvcrush_oracle_scores_append.argtypes = [i32] * 8 + [f64, vp, vp, vp]
        L.kvcrush_oracle_compact_cache.argtypes = [i32] * 8 + [vp] * 7
        L.kvcrush_oracle_topk.argtypes = [vp, i32, i32, vp]
        L.kvcrush_oracle_splitmix64.argtypes = [u64, i32, vp]
        L.kvcrush_oracle_splitmix64.restype = None
        L.kvcrush_oracle_bits.argtypes = [i32, i32, i32, vp, vp]
        L.kvcrush_oracle_group.argtypes = [i32, i32, vp, vp, i32, i32, u64, i32, vp, vp, vp]
        L.kvcrush_oracle_select.argtypes = [i32] * 7 + [u64, vp, vp, vp, vp, vp]
        L.kvcrush_oracle_select_protected.argtypes = [i32] * 9 + [u64, vp, vp, vp, vp, vp]
        L.kvcrush_oracle_select_units.argtypes = [i32] * 10 + [u64, vp, vp, vp, vp, vp]
        L.kvcrush_oracle_compact.argtypes = [i32] * 6 + [vp, vp, vp, vp, i32, vp, vp]
        _lib = L
    return _lib


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float16:
        return F16
    raise TypeError(f"oracle handles float32, bfloat16 and float16, got {t.dtype}")


def _cpu(t: torch.Tensor) -> torch.Tensor:
    assert t.device.type == "cpu", "the oracle reads host memory only"
    return t.contiguous()


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def words_for(Hs: int) -> int:
    return (Hs + 63) // 64


def head_colsums(q_head, k_head, row_begin=0, row_end=None, want_lse=False, scale=0.0):
    """Received attention for one head over query rows [row_begin, row_end).

    q_head, k_head: [S, D].  Returns float64 [S] (and float64 lse [S], zero
    outside the row range, when want_lse)."""
    q_head, k_head = _cpu(q_head), _cpu(k_head)
    S, D = q_head.shape
    row_end = S if row_end is None else row_end
    c = torch.zeros(S, dtype=torch.float64)
    lse = torch.zeros(S, dtype=torch.float64) if want_lse else None
    rc = lib().kvcrush_oracle_head_colsums(S, D, _dtype_code(q_head), _ptr(q_head), _ptr(k_head),
                                           row_begin, row_end, scale, _ptr(c), _ptr(lse))
    _check(rc, "head_colsums")
    return (c, lse) if want_lse else c


def scores(q, k, reduce_groups: bool, want_lse=False, threads: int = 1, window: int = 0, scale: float = 0.0):
    """scores [B,Hs,S] fp32 from q [B,Hq,S,D], k [B,Hkv,S,D].

    window = W > 0: only the last min(W, S) query rows contribute (lse rows
    before the window are zero).  scale: factor on the dot products (0: 1/sqrt(D)).

    threads > 1 spreads independent (batch, head) units of the unchanged
    single-threaded routine over host threads (the foreign call releases the
    GIL); the group sum is then formed here in float64, heads ascending,
    rounded once, exactly as the C++ whole-tensor routine does."""
    q, k = _cpu(q), _cpu(k)
    B, Hq, S, D = q.shape
    Hkv = k.shape[1]
    assert k.shape == (B, Hkv, S, D) and Hq % Hkv == 0 and q.dtype == k.dtype
    G = Hq // Hkv
    Hs = Hkv if reduce_groups else Hq
    if threads <= 1:
        out = torch.empty(B, Hs, S, dtype=torch.float32)
        lse = torch.empty(B, Hq, S, dtype=torch.float32) if want_lse else None
        rc = lib().kvcrush_oracle_scores(B, Hq, Hkv, S, D, _dtype_code(q), int(reduce_groups), window, scale,
                                         _ptr(q), _ptr(k), _ptr(out), _ptr(lse))
        _check(rc, "scores")
        return (out, lse) if want_lse else out

    row_begin = 0 if window == 0 or window >= S else S - window
    units = [(b, h) for b in range(B) for h in range(Hq)]
    with ThreadPoolExecutor(max_workers=threads) as ex:
        res = list(ex.map(lambda u: head_colsums(q[u[0], u[1]], k[u[0], u[1] // G], row_begin, S,
                                                 want_lse=True, scale=scale), units))
    c = torch.stack([r[0] for r in res]).view(B, Hq, S)
    lse = torch.stack([r[1] for r in res]).view(B, Hq, S).to(torch.float32)
    if reduce_groups:
        acc = torch.zeros(B, Hkv, S, dtype=torch.float64)
        for hh in range(G):  # ascending head order within each group
            acc = acc + c[:, hh::G, :]
        out = acc.to(torch.float32)
    else:
        out = c.to(torch.float32)
    return (out, lse) if want_lse else out


def scores_append(q_new, k_cache, scores_cache, S: int, reduce_groups: bool, scale: float = 0.0):
    """One decoding step, in place on scores_cache [B,Hs,capacity] (fp32): the new token's
    queries q_new [B,Hq,D] attend to the first S tokens of k_cache [B,Hkv,capacity,D]."""
    q_new, k_cache = _cpu(q_new), _cpu(k_cache)
    assert scores_cache.device.type == "cpu" and scores_cache.is_contiguous() and scores_cache.dtype == torch.float32
    B, Hq, D = q_new.shape
    Hkv, cap = k_cache.shape[1], k_cache.shape[2]
    assert scores_cache.shape == (B, Hkv if reduce_groups else Hq, cap)
    rc = lib().kvcrush_oracle_scores_append(B, Hq, Hkv, S, cap, D, _dtype_code(q_new), int(reduce_groups), scale,
                                            _ptr(q_new), _ptr(k_cache), _ptr(scores_cache))
    _check(rc, "scores_append")
    return scores_cache


def compact_cache(k, v, scores_t, idx, k_out, v_out, scores_out):
    """Eviction on capacity-strided caches: k, v [B,Hkv,cap_src,D], scores_t [B,Hs,cap_src] ->
    first idx.shape[1] tokens of k_out, v_out [B,Hkv,cap_dst,D], scores_out [B,Hs,cap_dst] (in place)."""
    k, v, sc, idx = _cpu(k), _cpu(v), _cpu(scores_t), _cpu(idx.to(torch.int32))
    for t in (k_out, v_out, scores_out):
        assert t.device.type == "cpu" and t.is_contiguous()
    B, Hkv, cap_src, D = k.shape
    rc = lib().kvcrush_oracle_compact_cache(B, Hkv, sc.shape[1], D, _dtype_code(k), cap_src, k_out.shape[2],
                                            idx.shape[1], _ptr(k), _ptr(v), _ptr(sc), _ptr(idx), _ptr(k_out),
                                            _ptr(v_out), _ptr(scores_out))
    _check(rc, "compact_cache")
    return k_out, v_out, scores_out


def maxpool(scores_t, kernel: int):
    """Centred 1-D max pool (odd kernel, -inf padding) along the last axis of fp32 scores."""
    sc = _cpu(scores_t.to(torch.float32))
    S = sc.shape[-1]
    out = torch.empty_like(sc)
    _check(lib().kvcrush_oracle_maxpool(sc.numel() // S, S, kernel, _ptr(sc), _ptr(out)), "maxpool")
    return out


def topk(v, k: int):
    v = _cpu(v.to(torch.float32))
    out = torch.empty(k, dtype=torch.int32)
    _check(lib().kvcrush_oracle_topk(_ptr(v), v.numel(), k, _ptr(out)), "topk")
    return out


def splitmix64(seed: int, count: int):
    out = torch.empty(count, dtype=torch.int64)
    lib().kvcrush_oracle_splitmix64(ctypes.c_uint64(seed & (2**64 - 1)), count, _ptr(out))
    return [int(x) & (2**64 - 1) for x in out.tolist()]


def bits(scores_1seq, kbit: int):
    """scores_1seq [Hs,S] fp32 -> packed head-behaviour words [S,W] (int64 storage)."""
    sc = _cpu(scores_1seq.to(torch.float32))
    Hs, S = sc.shape
    out = torch.empty(S, words_for(Hs), dtype=torch.int64)
    _check(lib().kvcrush_oracle_bits(Hs, S, kbit, _ptr(sc), _ptr(out)), "bits")
    return out


def group(Hs, bits_1seq, is_important, Br, anchor="alternating", anchor_seed=0, batch_index=0,
          anchor_explicit=None):
    """Alg. 2 on one sequence.  Returns (reps int32 [Br] in bucket order, anchor words)."""
    bw = _cpu(bits_1seq.to(torch.int64))
    S, W = bw.shape
    assert W == words_for(Hs)
    imp = _cpu(is_important.to(torch.uint8))
    reps = torch.empty(max(Br, 1), dtype=torch.int32)
    anc = torch.zeros(W, dtype=torch.int64)
    ae = None if anchor_explicit is None else _cpu(anchor_explicit.to(torch.int64))
    rc = lib().kvcrush_oracle_group(Hs, S, _ptr(bw), _ptr(imp), Br, ANCHORS[anchor],
                                    ctypes.c_uint64(anchor_seed & (2**64 - 1)), batch_index,
                                    _ptr(ae), _ptr(reps), _ptr(anc))
    _check(rc, "group")
    return reps[:Br], anc


def select(scores_t, budget, n_important, bit_topk=0, anchor="alternating", anchor_seed=0,
           anchor_bits=None, n_sink=0, n_recent=0):
    """Stages 2-4.  scores_t [B,Hs,S] fp32 -> (idx int32 [B,budget], kind uint8, bits int64 [B,S,W]).
    n_sink / n_recent: tokens at the two ends that are always kept (kind 2); the
    middle is compressed to budget - n_sink - n_recent tokens."""
    sc = _cpu(scores_t.to(torch.float32))
    B, Hs, S = sc.shape
    W = words_for(Hs)
    idx = torch.empty(B, budget, dtype=torch.int32)
    kind = torch.empty(B, budget, dtype=torch.uint8)
    bw = torch.empty(B, S, W, dtype=torch.int64)
    ab = None if anchor_bits is None else _cpu(anchor_bits.to(torch.int64))
    if n_sink or n_recent:
        rc = lib().kvcrush_oracle_select_protected(B, Hs, S, budget, n_important, bit_topk, n_sink, n_recent,
                                                   ANCHORS[anchor], ctypes.c_uint64(anchor_seed & (2**64 - 1)),
                                                   _ptr(ab), _ptr(sc), _ptr(idx), _ptr(kind), _ptr(bw))
    else:
        rc = lib().kvcrush_oracle_select(B, Hs, S, budget, n_important, bit_topk, ANCHORS[anchor],
                                         ctypes.c_uint64(anchor_seed & (2**64 - 1)), _ptr(ab), _ptr(sc),
                                         _ptr(idx), _ptr(kind), _ptr(bw))
    _check(rc, "select")
    return idx, kind, bw


def select_units(scores_t, unit, budget, n_important, bit_topk=0, anchor="alternating", anchor_seed=0,
                 anchor_bits=None, n_sink=0, n_recent=0):
    """Chunk- / page-level stages 2-4: the unit of selection is `unit` consecutive tokens.
    Returns (idx int32 [B,budget] tokens, kind uint8 [B,budget], unit bits int64 [B,Nu,Wu])."""
    sc = _cpu(scores_t.to(torch.float32))
    B, Hs, S = sc.shape
    Nu = max((S - n_sink - n_recent) // unit, 0)
    Wu = words_for(Hs * unit)
    idx = torch.empty(B, budget, dtype=torch.int32)
    kind = torch.empty(B, budget, dtype=torch.uint8)
    ub = torch.zeros(B, Nu, Wu, dtype=torch.int64)
    ab = None if anchor_bits is None else _cpu(anchor_bits.to(torch.int64))
    rc = lib().kvcrush_oracle_select_units(B, Hs, S, unit, budget, n_important, bit_topk, n_sink, n_recent,
                                           ANCHORS[anchor], ctypes.c_uint64(anchor_seed & (2**64 - 1)), _ptr(ab),
                                           _ptr(sc), _ptr(idx), _ptr(kind), _ptr(ub))
    _check(rc, "select_units")
    return idx, kind, ub


def compact(k, v, idx, block_table=None, block_size=16, dense_shape=None):
    """Stage 5.  Dense k, v [B,Hkv,S,D]; or paged pools [n_blocks,block_size,Hkv,D]
    with block_table [B,S/block_size] and dense_shape=(B,Hkv,S,D)."""
    k, v, idx = _cpu(k), _cpu(v), _cpu(idx.to(torch.int32))
    if block_table is None:
        B, Hkv, S, D = k.shape
    else:
        B, Hkv, S, D = dense_shape
        block_table = _cpu(block_table.to(torch.int32))
    budget = idx.shape[1]
    ko = torch.empty(B, Hkv, budget, D, dtype=k.dtype)
    vo = torch.empty(B, Hkv, budget, D, dtype=v.dtype)
    rc = lib().kvcrush_oracle_compact(B, Hkv, S, D, _dtype_code(k), budget, _ptr(k), _ptr(v),
                                      _ptr(idx), _ptr(block_table), block_size, _ptr(ko), _ptr(vo))
    _check(rc, "compact")
    return ko, vo
