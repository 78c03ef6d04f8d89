"""The selection entry point for callers that cannot allocate (kvcrush_select_static: the
library's own fixed scratch array instead of a workspace) against kvcrush_select on the same
inputs, bit for bit, on two calls in a row, the second with a smaller input."""
import pytest
import torch

from paper_2503_00022_amd import inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kv():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2503_00022_amd import binding, build
    build.ensure_built()
    binding.load()
    return binding


def both_ways(kv, B, Hs, S, budget, n_imp, anchor, seed, **kw):
    sc = inputs.make_scores(B, Hs, S, seed=seed, ties=True).cuda()
    ref_idx, ref_kind, ref_bits = kv.kvcrush_select(sc, budget, n_imp, 0, anchor, 5, want_bits=True, **kw)
    args = kv.make_select_args(B, Hs, S, budget, n_imp, 0, anchor, 5, **kw)
    assert kv.kvcrush_select_workspace(args) <= kv.SELECT_STATIC_MAX_BYTES
    idx = torch.full_like(ref_idx, -7)
    kind = torch.full_like(ref_kind, 9)
    bits = torch.full_like(ref_bits, -1)
    before = torch.cuda.memory_allocated()
    kv.kvcrush_select_static(args, sc, idx, kind, bits)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    assert torch.equal(idx, ref_idx) and torch.equal(kind, ref_kind) and torch.equal(bits, ref_bits)
    # without kinds and bit words (the bit words then live in the scratch array)
    idx2 = torch.full_like(ref_idx, -7)
    kv.kvcrush_select_static(args, sc, idx2)
    torch.cuda.synchronize()
    assert torch.equal(idx2, ref_idx)


def test_static_scratch_selection_equals_the_workspace_one_twice_in_a_row(kv):
    print("static-scratch select: config-3 sizes, then a smaller ragged one", flush=True)
    both_ways(kv, 1, 8, 16384, 4096, 3072, "mean", seed=1)
    both_ways(kv, 2, 5, 1000, 300, 100, "alternating", seed=2, n_sink=3, n_recent=17)
    both_ways(kv, 1, 8, 4096, 1024, 768, "random", seed=3, unit=16)


def test_static_scratch_selection_rejects_what_does_not_fit(kv):
    print("static-scratch select: a problem beyond the array's size", flush=True)
    B, Hs, S, budget = 16, 8, 32768, 1024
    args = kv.make_select_args(B, Hs, S, budget, 768)
    assert kv.kvcrush_select_workspace(args) > kv.SELECT_STATIC_MAX_BYTES
    sc = torch.zeros(1, device="cuda")   # never read: the size check comes first
    idx = torch.zeros(B, budget, dtype=torch.int32, device="cuda")
    with pytest.raises(kv.KVCrushError) as e:
        kv.kvcrush_select_static(args, sc, idx)
    assert e.value.status == kv.ERR_WORKSPACE
