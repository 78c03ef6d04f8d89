"""Call sequences over the C ABI for the two ways the library is used: compressing a
layer's cache after prefill, and keeping a compressed cache while decoding.

Nothing here computes: the classes own the buffers (outputs, workspaces, the
ping-pong halves of a decoding cache), pass device pointers to the library and
move the new token's K/V row into its slot.  All work is enqueued on the current
HIP stream; nothing synchronises.
"""
from __future__ import annotations

import torch

from . import binding as kv


class LayerCompressor:
    """scores -> select -> compact for layers of one fixed shape, with every buffer allocated once.

    q [B,Hq,S,D], k and v [B,Hkv,S,D] on the GPU; returns (idx, k_out, v_out) that are overwritten
    by the next call.  `window` / `pool` give the observation-window scoring with max pooling,
    `n_sink` / `n_recent` the protected ends, `unit` chunk- or page-level selection."""

    def __init__(self, B, Hq, Hkv, S, D, dtype, budget, n_important, *, reduce_groups=True, anchor="alternating",
                 anchor_seed=0, bit_topk=0, n_sink=0, n_recent=0, unit=0, window=0, pool=0, scale=0.0,
                 device="cuda"):
        self.reduce_groups, self.window, self.pool, self.scale = reduce_groups, window, pool, scale
        self.budget, self.n_important, self.bit_topk = budget, n_important, bit_topk
        self.anchor, self.anchor_seed = anchor, anchor_seed
        self.n_sink, self.n_recent, self.unit = n_sink, n_recent, unit
        Hs = Hkv if reduce_groups else Hq
        dev = torch.device(device)
        probe = kv.Shape(B, Hq, Hkv, S, D, {torch.float32: kv.F32, torch.bfloat16: kv.BF16, torch.float16: kv.F16}[dtype],
                         int(reduce_groups), window, scale)
        self.scores = torch.empty(B, Hs, S, dtype=torch.float32, device=dev)
        self.pooled = torch.empty_like(self.scores) if pool else None
        self.scores_ws = torch.empty(max(kv.kvcrush_scores_workspace(probe), 16), dtype=torch.uint8, device=dev)
        args = kv.make_select_args(B, Hs, S, budget, n_important, bit_topk, anchor, anchor_seed, None, n_sink, n_recent,
                                   0, unit)
        need = kv.kvcrush_select_workspace(args)
        if need == 0 and S - n_sink - n_recent > 0:
            raise ValueError("inconsistent or unsupported selection arguments")
        self.select_ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
        self.idx = torch.empty(B, budget, dtype=torch.int32, device=dev)
        self.k_out = torch.empty(B, Hkv, budget, D, dtype=dtype, device=dev)
        self.v_out = torch.empty_like(self.k_out)
        self._graph = None

    def run(self, q, k, v, lse=None, anchor_seed=None):
        """Enqueue one layer.  `lse` [B,Hq,S] fp32: the attention kernel's row normalisers, if it kept them."""
        kv.kvcrush_scores(q, k, self.reduce_groups, lse=lse, scores=self.scores, workspace=self.scores_ws,
                          window=self.window, scale=self.scale)
        sc = self.scores
        if self.pool:
            sc = kv.kvcrush_pool_scores(self.scores, self.pool, out=self.pooled)
        kv.kvcrush_select(sc, self.budget, self.n_important, self.bit_topk, self.anchor,
                          self.anchor_seed if anchor_seed is None else anchor_seed, want_kind=False, idx=self.idx,
                          workspace=self.select_ws, n_sink=self.n_sink, n_recent=self.n_recent, unit=self.unit)
        kv.kvcrush_compact(k, v, self.idx, k_out=self.k_out, v_out=self.v_out, validate=False)
        return self.idx, self.k_out, self.v_out

    def capture(self, q, k, v, lse=None):
        """Capture run() on these (static) input tensors in a HIP graph; replay() then re-runs it
        on whatever the tensors hold.  The entry points allocate nothing, so they capture as they are."""
        self.run(q, k, v, lse)                      # warm-up outside the capture
        torch.cuda.synchronize()
        self._graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            with torch.cuda.graph(self._graph, stream=side):
                self.run(q, k, v, lse)
        torch.cuda.synchronize()
        return self

    def replay(self):
        if self._graph is None:
            raise RuntimeError("capture() first")
        self._graph.replay()
        return self.idx, self.k_out, self.v_out


class DecodeCache:
    """A compressed KV cache that lives through decoding: K, V and the running scores in
    capacity-strided buffers, one more query row added to the scores per generated token,
    eviction back to `budget` tokens whenever the buffer is full (two buffer sets, swapped)."""

    def __init__(self, k, v, scores, budget, n_important, capacity, *, reduce_groups=True, anchor="alternating",
                 anchor_seed=0, bit_topk=0, n_sink=0, n_recent=0, scale=0.0):
        """k, v [B,Hkv,n,D] and scores [B,Hs,n]: a cache and its accumulated scores (for instance the
        outputs of a LayerCompressor with the scores gathered by kvcrush_compact_cache), n <= capacity."""
        B, Hkv, n, D = k.shape
        Hs = scores.shape[1]
        if capacity <= budget or n > capacity:
            raise ValueError("capacity must exceed the budget and hold the initial cache")
        self.budget, self.n_important, self.bit_topk = budget, n_important, bit_topk
        self.anchor, self.anchor_seed, self.n_sink, self.n_recent = anchor, anchor_seed, n_sink, n_recent
        self.reduce_groups, self.scale, self.capacity, self.n = reduce_groups, scale, capacity, n
        dev = k.device
        mk = lambda *shape, dtype: torch.zeros(*shape, dtype=dtype, device=dev)
        self._sets = [(mk(B, Hkv, capacity, D, dtype=k.dtype), mk(B, Hkv, capacity, D, dtype=k.dtype),
                       mk(B, Hs, capacity, dtype=torch.float32)) for _ in range(2)]
        self._cur = 0
        self.k[:, :, :n].copy_(k)
        self.v[:, :, :n].copy_(v)
        self.scores[:, :, :n].copy_(scores)
        self._append_ws = None                       # sized at the first append, which brings the query head count
        self._select_ws = torch.empty(max(kv.kvcrush_select_workspace(kv.make_select_args(
            B, Hs, capacity, budget, n_important, bit_topk, anchor, anchor_seed, None, n_sink, n_recent, capacity)), 16),
            dtype=torch.uint8, device=dev)
        self._idx = torch.empty(B, budget, dtype=torch.int32, device=dev)
        self.evictions = 0

    k = property(lambda self: self._sets[self._cur][0])
    v = property(lambda self: self._sets[self._cur][1])
    scores = property(lambda self: self._sets[self._cur][2])

    def evict(self):
        """Select `budget` of the n valid tokens and move them (with their scores) to the other buffer set."""
        kv.kvcrush_select(self.scores, self.budget, self.n_important, self.bit_topk, self.anchor, self.anchor_seed,
                          want_kind=False, idx=self._idx, workspace=self._select_ws, n_sink=self.n_sink,
                          n_recent=self.n_recent, valid_len=self.n)
        other = self._sets[1 - self._cur]
        kv.kvcrush_compact_cache(self.k, self.v, self.scores, self._idx, *other)
        self._cur, self.n = 1 - self._cur, self.budget
        self.evictions += 1
        return self._idx

    def append(self, q_new, k_new, v_new):
        """One generated token: q_new [B,Hq,D], k_new and v_new [B,Hkv,D].  Evicts first if the buffer is full."""
        if self.n == self.capacity:
            self.evict()
        self.k[:, :, self.n].copy_(k_new)
        self.v[:, :, self.n].copy_(v_new)
        self.n += 1
        if self._append_ws is None:
            B, Hq, D = q_new.shape
            probe = kv.Shape(B, Hq, self.k.shape[1], self.capacity, D, kv._dtype_code(q_new), int(self.reduce_groups),
                             0, self.scale)
            self._append_ws = torch.empty(max(kv.kvcrush_scores_append_workspace(probe, self.capacity), 16),
                                          dtype=torch.uint8, device=q_new.device)
        kv.kvcrush_scores_append(q_new, self.k, self.scores, self.n, self.reduce_groups, workspace=self._append_ws,
                                 scale=self.scale)
        return self.n
