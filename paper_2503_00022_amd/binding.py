"""Thin ctypes binding over libkvcrush.so: same names as the C ABI
(include/kvcrush.h), argument marshalling only.  torch is used for device
memory and the current HIP stream; every computation happens in the library's
kernels.  There is no fallback: if the library is missing or a call fails, an
exception is raised.
"""
from __future__ import annotations

import ctypes
import os

import torch

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libkvcrush.so")

F32, BF16, F16 = 0, 1, 2
ANCHORS = {"random": 0, "mean": 1, "alternating": 2, "explicit": 3}
OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP = range(5)

EXPORTS = (
    "kvcrush_scores_workspace", "kvcrush_scores", "kvcrush_row_lse_workspace", "kvcrush_row_lse",
    "kvcrush_pool_scores",
    "kvcrush_select_workspace", "kvcrush_select", "kvcrush_select_static", "kvcrush_compact", "kvcrush_scores_append_workspace",
    "kvcrush_scores_append", "kvcrush_compact_cache", "kvcrush_compact_block_table", "kvcrush_status_string",
    "kvcrush_version",
)


class KVCrushError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {status_string(status)} (status {status})")


class Shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("B", "Hq", "Hkv", "S", "D", "dtype", "reduce_groups",
                                                 "obs_window")] + [("softmax_scale", ctypes.c_float),
                                                                   ("q_stride", ctypes.c_int64 * 3),
                                                                   ("k_stride", ctypes.c_int64 * 3)]


class SelectArgs(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("B", "Hs", "S", "budget", "n_important", "bit_topk", "anchor",
                                                 "score_stride", "n_sink", "n_recent", "unit")] + [
        ("anchor_seed", ctypes.c_uint64), ("anchor_bits", ctypes.c_void_p)]


_lib = None


def load() -> ctypes.CDLL:
    """Load the library built by `paper_2503_00022_amd.build` (never builds, never falls back)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2503_00022_amd.build` "
                "(or __graft_entry__.build()); there is no CPU fallback")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        L.kvcrush_scores_workspace.argtypes = [ctypes.POINTER(Shape)]
        L.kvcrush_scores_workspace.restype = sz
        L.kvcrush_scores.argtypes = [ctypes.POINTER(Shape), vp, vp, vp, vp, vp, sz, vp]
        L.kvcrush_scores.restype = ctypes.c_int
        L.kvcrush_row_lse_workspace.argtypes = [ctypes.POINTER(Shape)]
        L.kvcrush_row_lse_workspace.restype = sz
        L.kvcrush_row_lse.argtypes = [ctypes.POINTER(Shape), vp, vp, vp, vp, sz, vp]
        L.kvcrush_row_lse.restype = ctypes.c_int
        L.kvcrush_pool_scores.argtypes = [i32, i32, i32, vp, vp, vp]
        L.kvcrush_pool_scores.restype = ctypes.c_int
        L.kvcrush_select_workspace.argtypes = [ctypes.POINTER(SelectArgs)]
        L.kvcrush_select_workspace.restype = sz
        L.kvcrush_select.argtypes = [ctypes.POINTER(SelectArgs), vp, vp, vp, vp, vp, sz, vp]
        L.kvcrush_select.restype = ctypes.c_int
        L.kvcrush_select_static.argtypes = [ctypes.POINTER(SelectArgs), vp, vp, vp, vp, vp]
        L.kvcrush_select_static.restype = ctypes.c_int
        L.kvcrush_compact.argtypes = [i32] * 6 + [vp, vp, vp, vp, i32, vp, vp, vp]
        L.kvcrush_compact.restype = ctypes.c_int
        L.kvcrush_scores_append_workspace.argtypes = [ctypes.POINTER(Shape), i32]
        L.kvcrush_scores_append_workspace.restype = sz
        L.kvcrush_scores_append.argtypes = [ctypes.POINTER(Shape), i32, vp, vp, vp, vp, i32, vp, vp, sz, vp]
        L.kvcrush_scores_append.restype = ctypes.c_int
        L.kvcrush_compact_cache.argtypes = [i32] * 8 + [vp] * 8
        L.kvcrush_compact_cache.restype = ctypes.c_int
        L.kvcrush_compact_block_table.argtypes = [i32] * 4 + [vp] * 4
        L.kvcrush_compact_block_table.restype = ctypes.c_int
        L.kvcrush_status_string.argtypes = [ctypes.c_int]
        L.kvcrush_status_string.restype = ctypes.c_char_p
        L.kvcrush_version.restype = i32
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return load().kvcrush_status_string(status).decode()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float16:
        return F16
    raise TypeError(f"kvcrush handles float32, bfloat16 and float16, got {t.dtype}")


def _dev(t: torch.Tensor, name: str) -> torch.Tensor:
    if t.device.type != "cuda":
        raise ValueError(f"{name} must live in GPU memory")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t


def _dev_rows(t: torch.Tensor, name: str) -> torch.Tensor:
    """A [B,H,S,D] tensor or view on the GPU whose D values are contiguous (any other strides)."""
    if t.device.type != "cuda":
        raise ValueError(f"{name} must live in GPU memory")
    if t.dim() != 4 or (t.shape[3] > 1 and t.stride(3) != 1):
        raise ValueError(f"{name} must be [B,H,S,D] with the D values contiguous")
    return t


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _check(status: int, what: str):
    if status != OK:
        raise KVCrushError(status, what)


def make_shape(q: torch.Tensor, k: torch.Tensor, reduce_groups: bool, window: int = 0, scale: float = 0.0) -> Shape:
    B, Hq, S, D = q.shape
    shape = Shape(B, Hq, k.shape[1], S, D, _dtype_code(q), int(bool(reduce_groups)), int(window), float(scale))
    for t, field in ((q, shape.q_stride), (k, shape.k_stride)):
        if not t.is_contiguous():                     # views (a transposed projection output, a slice of a
            field[:] = list(t.stride()[:3])           # padded buffer) are read in place, never copied
    return shape


def kvcrush_scores_workspace(shape: Shape) -> int:
    return int(load().kvcrush_scores_workspace(ctypes.byref(shape)))


def kvcrush_scores(q, k, reduce_groups: bool, lse=None, scores=None, workspace=None, stream=None, window=0,
                   scale=0.0):
    """q [B,Hq,S,D], k [B,Hkv,S,D] on the GPU -> scores [B,Hs,S] fp32.
    window = W > 0 restricts the contributing queries to the last min(W, S).
    scale: factor on Q.K before the softmax (0: 1/sqrt(D)).
    Returns (scores, workspace); the workspace's first B*Hq*S floats hold the
    row log-sum-exps when `lse` was not supplied.
    q and k may be views with any sequence, head and token strides (D contiguous)."""
    q, k = _dev_rows(q, "q"), _dev_rows(k, "k")
    if q.dtype != k.dtype or q.dim() != 4 or k.dim() != 4 or q.shape[0] != k.shape[0] \
            or q.shape[2:] != k.shape[2:]:
        raise ValueError("q and k must be [B,H,S,D] tensors of one dtype with matching B, S, D")
    shape = make_shape(q, k, reduce_groups, window, scale)
    Hs = shape.Hkv if reduce_groups else shape.Hq
    if scores is None:
        scores = torch.empty(shape.B, Hs, shape.S, dtype=torch.float32, device=q.device)
    need = kvcrush_scores_workspace(shape)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    if lse is not None:
        lse = _dev(lse, "lse")
        if lse.dtype != torch.float32 or tuple(lse.shape) != (shape.B, shape.Hq, shape.S):
            raise ValueError("lse must be fp32 [B,Hq,S]")
    st = load().kvcrush_scores(ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(lse), _ptr(_dev(scores, "scores")),
                               _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream(stream))
    _check(st, "kvcrush_scores")
    return scores, workspace


def kvcrush_row_lse_workspace(shape: Shape) -> int:
    return int(load().kvcrush_row_lse_workspace(ctypes.byref(shape)))


def kvcrush_row_lse(q, k, lse_out=None, stream=None, window=0, workspace="auto", scale=0.0):
    """q [B,Hq,S,D], k [B,Hkv,S,D] on the GPU -> natural-log row normalisers fp32 [B,Hq,S]
    (with window = W > 0 only the rows of the last min(W, S) queries are defined).
    workspace: a uint8 tensor, None (run without scratch memory) or "auto" (allocate what
    kvcrush_row_lse_workspace asks for)."""
    q, k = _dev_rows(q, "q"), _dev_rows(k, "k")
    shape = make_shape(q, k, False, window, scale)
    if lse_out is None:
        lse_out = torch.empty(shape.B, shape.Hq, shape.S, dtype=torch.float32, device=q.device)
    if isinstance(workspace, str):
        workspace = torch.empty(max(kvcrush_row_lse_workspace(shape), 16), dtype=torch.uint8, device=q.device)
    st = load().kvcrush_row_lse(ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(_dev(lse_out, "lse_out")),
                                _ptr(workspace), 0 if workspace is None else workspace.numel(),
                                _stream(stream))
    _check(st, "kvcrush_row_lse")
    return lse_out


def kvcrush_pool_scores(scores, kernel: int, out=None, stream=None):
    """Centred sliding maximum of width `kernel` (odd) along the last axis of fp32 scores."""
    scores = _dev(scores, "scores")
    if scores.dtype != torch.float32:
        raise ValueError("scores must be fp32")
    if out is None:
        out = torch.empty_like(scores)
    S = scores.shape[-1]
    st = load().kvcrush_pool_scores(scores.numel() // S, S, kernel, _ptr(scores), _ptr(_dev(out, "out")),
                                    _stream(stream))
    _check(st, "kvcrush_pool_scores")
    return out


def lse_from_workspace(workspace: torch.Tensor, B: int, Hq: int, S: int) -> torch.Tensor:
    return workspace[: B * Hq * S * 4].view(torch.float32).view(B, Hq, S)


def make_select_args(B, Hs, S, budget, n_important, bit_topk=0, anchor="alternating", anchor_seed=0,
                     anchor_bits=None, n_sink=0, n_recent=0, score_stride=0, unit=0) -> SelectArgs:
    return SelectArgs(B, Hs, S, budget, n_important, bit_topk, ANCHORS[anchor] if isinstance(anchor, str) else anchor,
                      score_stride, n_sink, n_recent, unit, anchor_seed & (2**64 - 1),
                      None if anchor_bits is None else anchor_bits.data_ptr())


def kvcrush_select_workspace(args: SelectArgs) -> int:
    return int(load().kvcrush_select_workspace(ctypes.byref(args)))


def kvcrush_select(scores, budget, n_important, bit_topk=0, anchor="alternating", anchor_seed=0,
                   anchor_bits=None, want_kind=True, want_bits=False, idx=None, workspace=None, stream=None,
                   n_sink=0, n_recent=0, valid_len=None, unit=0):
    """scores [B,Hs,S] fp32 on the GPU -> (idx int32 [B,budget], kind uint8 | None, bits int64 [B,S,W] | None).
    n_sink / n_recent tokens at the two ends are always kept; the rest of the budget goes to the middle.
    valid_len: scores is a capacity-strided cache [B,Hs,capacity] of which the first valid_len tokens count."""
    scores = _dev(scores, "scores")
    if scores.dtype != torch.float32 or scores.dim() != 3:
        raise ValueError("scores must be fp32 [B,Hs,S]")
    B, Hs, S = scores.shape
    stride = 0
    if valid_len is not None:
        stride, S = S, int(valid_len)
    if anchor_bits is not None:
        anchor_bits = _dev(anchor_bits, "anchor_bits")
    args = make_select_args(B, Hs, S, budget, n_important, bit_topk, anchor, anchor_seed, anchor_bits,
                            n_sink, n_recent, stride, unit)
    dev = scores.device
    if idx is None:
        idx = torch.empty(B, budget, dtype=torch.int32, device=dev)
    kind = torch.empty(B, budget, dtype=torch.uint8, device=dev) if want_kind else None
    if unit > 1:   # one vector of Hs * unit bits per unit of the middle
        bits_shape = (B, max(S - n_sink - n_recent, 0) // unit, (Hs * unit + 63) // 64)
    else:
        bits_shape = (B, S, (Hs + 63) // 64)
    bits = torch.empty(bits_shape, dtype=torch.int64, device=dev) if want_bits else None
    if workspace is None:
        workspace = torch.empty(max(kvcrush_select_workspace(args), 16), dtype=torch.uint8, device=dev)
    st = load().kvcrush_select(ctypes.byref(args), _ptr(scores), _ptr(idx), _ptr(kind), _ptr(bits),
                               _ptr(workspace), workspace.numel(), _stream(stream))
    _check(st, "kvcrush_select")
    return idx, kind, bits


SELECT_STATIC_MAX_BYTES = 4 << 20   # KVCRUSH_SELECT_STATIC_MAX_BYTES


def kvcrush_select_static(args: SelectArgs, scores, idx, kind=None, bits=None, stream=None):
    """kvcrush_select on the library's own fixed scratch array: every buffer is the caller's, nothing
    is allocated here or in the library.  args from make_select_args; idx int32 [B,budget], kind uint8
    [B,budget] or None, bits int64 or None, all preallocated on the GPU."""
    st = load().kvcrush_select_static(ctypes.byref(args), _ptr(_dev(scores, "scores")), _ptr(_dev(idx, "idx")),
                                      _ptr(kind), _ptr(bits), _stream(stream))
    _check(st, "kvcrush_select_static")
    return idx, kind, bits


def kvcrush_compact(k, v, idx, block_table=None, block_size=16, dense_shape=None, k_out=None, v_out=None,
                    stream=None, validate=True):
    """Dense k, v [B,Hkv,S,D]; or paged pools [n_blocks,block_size,Hkv,D] with block_table
    [B,S/block_size] int32 and dense_shape=(B,Hkv,S,D).  Returns (k_out, v_out) [B,Hkv,budget,D]."""
    k, v, idx = _dev(k, "k"), _dev(v, "v"), _dev(idx, "idx")
    if idx.dtype != torch.int32 or k.dtype != v.dtype or k.shape != v.shape:
        raise ValueError("idx must be int32; k and v must match")
    if block_table is None:
        B, Hkv, S, D = k.shape
    else:
        B, Hkv, S, D = dense_shape
        block_table = _dev(block_table, "block_table")
        if block_table.dtype != torch.int32 or tuple(block_table.shape) != (B, S // block_size):
            raise ValueError("block_table must be int32 [B, S/block_size]")
        if tuple(k.shape[1:]) != (block_size, Hkv, D):
            raise ValueError("paged pools must be [n_blocks, block_size, Hkv, D]")
    budget = idx.shape[1]
    if idx.shape[0] != B:
        raise ValueError("idx must be [B,budget]")
    if validate:  # host-side bounds checks of the gather's index operands (synchronises)
        if budget and (int(idx.min()) < 0 or int(idx.max()) >= S):
            raise ValueError("idx out of range")
        if block_table is not None and (int(block_table.min()) < 0 or int(block_table.max()) >= k.shape[0]):
            raise ValueError("block_table names a block outside the pool")
    if k_out is None:
        k_out = torch.empty(B, Hkv, budget, D, dtype=k.dtype, device=k.device)
    if v_out is None:
        v_out = torch.empty(B, Hkv, budget, D, dtype=v.dtype, device=v.device)
    st = load().kvcrush_compact(B, Hkv, S, D, _dtype_code(k), budget, _ptr(k), _ptr(v), _ptr(idx),
                                _ptr(block_table), block_size, _ptr(_dev(k_out, "k_out")),
                                _ptr(_dev(v_out, "v_out")), _stream(stream))
    _check(st, "kvcrush_compact")
    return k_out, v_out


def kvcrush_scores_append_workspace(shape: Shape, capacity: int) -> int:
    return int(load().kvcrush_scores_append_workspace(ctypes.byref(shape), capacity))


def kvcrush_scores_append(q_new, k_cache, scores_cache, S: int, reduce_groups: bool, workspace=None, stream=None,
                          lengths=None, block_table=None, block_size=16, scale=0.0):
    """One decoding step, in place on scores_cache [B,Hs,capacity] fp32: the new token's queries
    q_new [B,Hq,D] attend to the first S tokens of k_cache [B,Hkv,capacity,D] (the new key included).
    lengths: optional int32 [B] on the GPU with each sequence's own valid length (S is then their bound).
    block_table: k_cache is then a paged pool [n_blocks,block_size,Hkv,D], block_table int32
    [B,capacity/block_size]."""
    q_new, k_cache, scores_cache = _dev(q_new, "q_new"), _dev(k_cache, "k_cache"), _dev(scores_cache, "scores_cache")
    if q_new.dim() != 3 or k_cache.dim() != 4 or q_new.dtype != k_cache.dtype or scores_cache.dtype != torch.float32:
        raise ValueError("q_new [B,Hq,D] and k_cache [B,Hkv,capacity,D] of one dtype, scores_cache fp32")
    B, Hq, D = q_new.shape
    if block_table is None:
        Hkv, cap = k_cache.shape[1], k_cache.shape[2]
        if k_cache.shape[0] != B or k_cache.shape[3] != D:
            raise ValueError("q_new and k_cache disagree on B or D")
    else:
        block_table = _dev(block_table, "block_table")
        Hkv, cap = k_cache.shape[2], block_table.shape[1] * block_size
        if block_table.dtype != torch.int32 or block_table.shape[0] != B or k_cache.shape[1] != block_size \
                or k_cache.shape[3] != D:
            raise ValueError("paged k_cache must be [n_blocks,block_size,Hkv,D] with block_table int32 [B,n]")
    if tuple(scores_cache.shape) != (B, Hkv if reduce_groups else Hq, cap):
        raise ValueError("scores_cache must be [B,Hs,capacity]")
    shape = Shape(B, Hq, Hkv, int(S), D, _dtype_code(q_new), int(bool(reduce_groups)), 0, float(scale))
    if workspace is None:
        workspace = torch.empty(max(kvcrush_scores_append_workspace(shape, cap), 16), dtype=torch.uint8,
                                device=q_new.device)
    if lengths is not None:
        lengths = _dev(lengths, "lengths")
        if lengths.dtype != torch.int32 or tuple(lengths.shape) != (B,):
            raise ValueError("lengths must be int32 [B]")
    st = load().kvcrush_scores_append(ctypes.byref(shape), cap, _ptr(lengths), _ptr(q_new), _ptr(k_cache),
                                      _ptr(block_table), block_size, _ptr(scores_cache), _ptr(workspace),
                                      workspace.numel(), _stream(stream))
    _check(st, "kvcrush_scores_append")
    return scores_cache


def kvcrush_compact_cache(k, v, scores, idx, k_out, v_out, scores_out, stream=None):
    """Eviction on capacity-strided caches: the tokens idx [B,budget] of k, v [B,Hkv,cap_src,D] and of
    scores [B,Hs,cap_src] move to the front of k_out, v_out [B,Hkv,cap_dst,D], scores_out [B,Hs,cap_dst]."""
    for name, t in (("k", k), ("v", v), ("scores", scores), ("idx", idx), ("k_out", k_out), ("v_out", v_out),
                    ("scores_out", scores_out)):
        _dev(t, name)
    if idx.dtype != torch.int32 or k.dtype != v.dtype or k.shape != v.shape or k_out.shape != v_out.shape \
            or k_out.dtype != k.dtype or scores.dtype != torch.float32 or scores_out.dtype != torch.float32:
        raise ValueError("idx int32; k, v, k_out, v_out of one dtype; scores fp32")
    B, Hkv, cap_src, D = k.shape
    cap_dst, Hs = k_out.shape[2], scores.shape[1]
    if tuple(scores.shape) != (B, Hs, cap_src) or tuple(scores_out.shape) != (B, Hs, cap_dst) \
            or tuple(k_out.shape) != (B, Hkv, cap_dst, D) or idx.shape[0] != B:
        raise ValueError("shapes of the source and destination caches do not match")
    st = load().kvcrush_compact_cache(B, Hkv, Hs, D, _dtype_code(k), cap_src, cap_dst, idx.shape[1], _ptr(k),
                                      _ptr(v), _ptr(scores), _ptr(idx), _ptr(k_out), _ptr(v_out),
                                      _ptr(scores_out), _stream(stream))
    _check(st, "kvcrush_compact_cache")
    return k_out, v_out, scores_out


def kvcrush_compact_block_table(idx, block_table, block_size: int, out=None, stream=None):
    """Page-level eviction on a paged pool: idx [B,budget] (whole blocks, from kvcrush_select with
    unit == block_size) and block_table [B,S/block_size] -> the kept blocks [B,budget/block_size]."""
    idx, block_table = _dev(idx, "idx"), _dev(block_table, "block_table")
    if idx.dtype != torch.int32 or block_table.dtype != torch.int32 or idx.shape[0] != block_table.shape[0]:
        raise ValueError("idx and block_table must be int32 with the same batch size")
    B, budget = idx.shape
    if out is None:
        out = torch.empty(B, budget // block_size, dtype=torch.int32, device=idx.device)
    st = load().kvcrush_compact_block_table(B, block_table.shape[1] * block_size, budget, block_size, _ptr(idx),
                                            _ptr(block_table), _ptr(_dev(out, "out")), _stream(stream))
    _check(st, "kvcrush_compact_block_table")
    return out


def kvcrush_version() -> int:
    return int(load().kvcrush_version())
