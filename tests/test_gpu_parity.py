"""Parity of the HIP path (through the C ABI) against the CPU oracle on the same
seeded inputs.  Bar: scores within 2e-3 relative per element; everything that
is integer or a copy (bits, indices, kinds, compacted K/V) bit-exact, the
selection being compared on the GPU's own score tensor."""
import os

import pytest
import torch

from paper_2503_00022_amd import inputs

pytestmark = pytest.mark.gpu

SCORE_RTOL = 2e-3
THREADS = min(16, os.cpu_count() or 1)


@pytest.fixture(scope="module")
def kv():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2503_00022_amd import binding, build
    build.ensure_built()  # compiles only when no library is there
    binding.load()        # the binding itself never builds and never falls back
    return binding


def rel_err(got, ref):
    ref = ref.double()
    return ((got.double().cpu() - ref).abs() / ref.abs().clamp_min(1e-12)).max().item()


def say(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------ stage 5
@pytest.mark.parametrize("B,Hkv,S,D,dtype,budget", [
    (2, 4, 96, 64, "bf16", 24), (1, 8, 1000, 128, "bf16", 333), (3, 2, 130, 128, "f32", 130),
    (1, 1, 17, 64, "f32", 1), (2, 8, 4096, 128, "bf16", 1024), (1, 3, 50, 64, "bf16", 0), (2, 2, 700, 128, "f16", 99),
    (2, 3, 70, 96, "f32", 33),      # 24 vectors a row: lanes per row not a power of two
    (1, 2, 40, 24, "bf16", 13),     # 3 vectors a row
    (1, 2, 50, 2048, "f32", 7),     # 8 KiB rows: more vectors than a workgroup has lanes
    (8, 8, 8192, 128, "bf16", 2048),  # config-4 size: the eight-rows-in-flight instantiation
])
def test_compact_dense(kv, oracle, B, Hkv, S, D, dtype, budget):
    say(f"compact dense B={B} Hkv={Hkv} S={S} D={D} {dtype} budget={budget}")
    w = inputs.Workload("t", B, Hkv, Hkv, S, D, dtype, budget, 0.5, "alternating", True)
    _, k, v = inputs.make_qkv(w, 3)
    g = torch.Generator().manual_seed(S + budget)
    idx = torch.stack([torch.randperm(S, generator=g)[:budget].sort().values for _ in range(B)]).int()
    ko, vo = kv.kvcrush_compact(k.cuda(), v.cuda(), idx.cuda())
    torch.cuda.synchronize()
    rk, rv = oracle.compact(k, v, idx)
    assert torch.equal(ko.cpu().view(torch.uint8), rk.view(torch.uint8))
    assert torch.equal(vo.cpu().view(torch.uint8), rv.view(torch.uint8))


@pytest.mark.parametrize("B,Hkv,S,D,budget,bs", [(3, 8, 128, 128, 40, 16), (1, 8, 32768, 128, 1024, 16),
                                                 (2, 2, 96, 64, 96, 32)])
def test_compact_paged(kv, oracle, B, Hkv, S, D, budget, bs):
    say(f"compact paged B={B} Hkv={Hkv} S={S} D={D} budget={budget} block={bs}")
    w = inputs.Workload("t", B, Hkv, Hkv, S, D, "bf16", budget, 0.25, "alternating", True, paged=True, block_size=bs)
    _, k, v = inputs.make_qkv(w, 4)
    bt = inputs.make_block_table(w, 9)
    kp, vp = inputs.to_paged(k, bt, bs), inputs.to_paged(v, bt, bs)
    g = torch.Generator().manual_seed(2)
    idx = torch.stack([torch.randperm(S, generator=g)[:budget].sort().values for _ in range(B)]).int()
    ko, vo = kv.kvcrush_compact(kp.cuda(), vp.cuda(), idx.cuda(), block_table=bt.cuda(), block_size=bs,
                                dense_shape=(B, Hkv, S, D))
    torch.cuda.synchronize()
    rk, rv = oracle.compact(kp, vp, idx, block_table=bt, block_size=bs, dense_shape=(B, Hkv, S, D))
    assert torch.equal(ko.cpu().view(torch.uint8), rk.view(torch.uint8))
    assert torch.equal(vo.cpu().view(torch.uint8), rv.view(torch.uint8))
    # and the paged gather equals the dense one
    dk, _ = oracle.compact(k, v, idx)
    assert torch.equal(ko.cpu().view(torch.uint8), dk.view(torch.uint8))


# --------------------------------------------------------------- stages 2-4
def check_select(kv, oracle, sc, budget, n_imp, kbit, anchor, seed=0, anchor_bits=None, n_sink=0, n_recent=0):
    ends = dict(n_sink=n_sink, n_recent=n_recent)
    idx, kind, bits = kv.kvcrush_select(sc.cuda(), budget, n_imp, kbit, anchor, seed,
                                        None if anchor_bits is None else anchor_bits.cuda(), want_bits=True, **ends)
    torch.cuda.synchronize()
    ridx, rkind, rbits = oracle.select(sc, budget, n_imp, kbit, anchor, seed, anchor_bits, **ends)
    assert torch.equal(bits.cpu(), rbits), "head-behaviour bit words differ"
    assert torch.equal(idx.cpu(), ridx), "retained indices differ"
    assert torch.equal(kind.cpu(), rkind), "important/representative labels differ"
    # same result when the caller does not ask for kinds or bits (bits then live in the workspace)
    idx2, kind2, bits2 = kv.kvcrush_select(sc.cuda(), budget, n_imp, kbit, anchor, seed,
                                           None if anchor_bits is None else anchor_bits.cuda(),
                                           want_kind=False, want_bits=False, **ends)
    torch.cuda.synchronize()
    assert kind2 is None and bits2 is None and torch.equal(idx2.cpu(), ridx)


@pytest.mark.parametrize("B,Hs,S,budget,n_imp,kbit,sink,recent,anchor", [
    (1, 8, 2000, 672, 384, 0, 32, 128, "alternating"),   # 32 initial + 512 middle + 128 recent (Table 1's layout)
    (2, 8, 1000, 300, 100, 0, 5, 17, "mean"),            # ragged ends: the middle starts off every alignment
    (1, 32, 4096, 1024, 512, 0, 4, 64, "random"),
    (2, 100, 700, 200, 50, 300, 3, 0, "mean"),           # sink only, two bit words, kbit > half the middle
    (1, 8, 333, 100, 0, 0, 0, 33, "alternating"),        # recent only, nothing important
    (1, 8, 16384, 4096, 2928, 0, 32, 128, "mean"),       # config-3 sizes
    (1, 4, 40000, 5000, 3000, 0, 64, 500, "random"),     # keys through the workspace
    (1, 8, 300, 300, 100, 0, 10, 20, "alternating"),     # budget == S
    (2, 8, 300, 30, 0, 0, 10, 20, "alternating"),        # the middle is dropped entirely
    (1, 8, 64, 64, 0, 0, 40, 24, "random"),              # there is no middle
    (1, 8, 65, 65, 0, 0, 1, 0, "alternating"),
])
def test_select_protected_ends(kv, oracle, B, Hs, S, budget, n_imp, kbit, sink, recent, anchor):
    say(f"select with protected ends B={B} Hs={Hs} S={S} budget={budget} n_imp={n_imp} sink={sink} recent={recent}")
    sc = inputs.make_scores(B, Hs, S, seed=S + sink + recent, ties=True)
    check_select(kv, oracle, sc, budget, n_imp, kbit, anchor, seed=11, n_sink=sink, n_recent=recent)


@pytest.mark.parametrize("B,Hs,S,unit,budget,n_imp,kbit,sink,recent,anchor", [
    (2, 8, 1024, 8, 256, 192, 0, 0, 0, "alternating"),        # chunks of 8 tokens: 64-bit vectors
    (1, 8, 4096, 16, 1024, 768, 0, 0, 0, "mean"),             # pages of 16: 128-bit vectors
    (1, 8, 32768, 32, 1024, 768, 0, 0, 0, "random"),          # config-5 sizes, pages of 32: 256-bit vectors
    (1, 8, 2080, 32, 672, 384, 0, 32, 128, "random"),         # Table 1: 32 initial + middle + 128 recent, page 32
    (2, 32, 2048, 32, 512, 256, 0, 0, 0, "alternating"),      # one bit per query head: 1024-bit vectors
    (2, 3, 900, 5, 400, 100, 500, 0, 0, "mean"),              # odd sizes; kbit > half: one-bits in the mean anchor
    (1, 4, 640, 4, 640, 160, 0, 0, 0, "mean"),                # budget == S
    (1, 4, 640, 4, 240, 0, 0, 40, 40, "alternating"),         # nothing important
    (1, 4, 640, 4, 240, 240, 0, 0, 0, "alternating"),         # no representatives: the paged top-k baseline
    (1, 12, 6000, 6, 1200, 600, 0, 0, 0, "random"),           # 72-bit vectors: a partly used second word
])
def test_select_units_matches_oracle(kv, oracle, B, Hs, S, unit, budget, n_imp, kbit, sink, recent, anchor):
    say(f"unit-level select B={B} Hs={Hs} S={S} unit={unit} budget={budget} n_imp={n_imp} sink={sink} recent={recent}")
    sc = inputs.make_scores(B, Hs, S, seed=S + unit, ties=True)
    ends = dict(n_sink=sink, n_recent=recent)
    idx, kind, bits = kv.kvcrush_select(sc.cuda(), budget, n_imp, kbit, anchor, 21, want_bits=True, unit=unit, **ends)
    torch.cuda.synchronize()
    ridx, rkind, rbits = oracle.select_units(sc, unit, budget, n_imp, kbit, anchor, 21, **ends)
    assert torch.equal(bits.cpu(), rbits), "unit bit vectors differ"
    assert torch.equal(idx.cpu(), ridx), "retained indices differ"
    assert torch.equal(kind.cpu(), rkind)
    idx2, _, _ = kv.kvcrush_select(sc.cuda(), budget, n_imp, kbit, anchor, 21, want_kind=False, unit=unit, **ends)
    torch.cuda.synchronize()
    assert torch.equal(idx2.cpu(), ridx)


def test_select_units_explicit_anchor(kv, oracle):
    say("unit-level select with a caller-supplied 192-bit anchor")
    B, Hs, S, unit = 2, 12, 1920, 16
    sc = inputs.make_scores(B, Hs, S, seed=77, ties=True)
    g = torch.Generator().manual_seed(3)
    anchor = torch.randint(-2**62, 2**62, (B, 3), generator=g, dtype=torch.int64)   # bits beyond 192 are ignored
    idx, kind, bits = kv.kvcrush_select(sc.cuda(), 480, 320, 0, "explicit", 0, anchor.cuda(), want_bits=True,
                                        unit=unit)
    torch.cuda.synchronize()
    ridx, rkind, rbits = oracle.select_units(sc, unit, 480, 320, 0, "explicit", 0, anchor)
    assert torch.equal(bits.cpu(), rbits) and torch.equal(idx.cpu(), ridx) and torch.equal(kind.cpu(), rkind)


@pytest.mark.parametrize("Hs,S,budget,n_imp,anchor", [(129, 700, 200, 120, "random"), (300, 1000, 300, 100, "mean"),
                                                       (1024, 512, 128, 64, "alternating")])
def test_select_many_score_rows(kv, oracle, Hs, S, budget, n_imp, anchor):
    """Token-level selection with more than 128 score rows (bit vectors of 3 to 16 words)."""
    say(f"select with Hs={Hs} score rows")
    sc = inputs.make_scores(1, Hs, S, seed=Hs, ties=True)
    check_select(kv, oracle, sc, budget, n_imp, S * 3 // 5 if anchor == "mean" else 0, anchor, seed=2)


def test_page_level_pipeline_on_a_paged_cache(kv, oracle):
    """Scores -> page-level selection (page = the cache's 16-token block) -> gather from the paged pool."""
    say("page-level selection on a paged cache")
    w = inputs.Workload("t", 1, 8, 2, 2048, 128, "bf16", 512, 0.25, "alternating", True, paged=True, block_size=16)
    seed = 31
    q, k, v = inputs.make_qkv(w, seed)
    sc, _ = kv.kvcrush_scores(q.cuda(), k.cuda(), True)
    idx, kind, _ = kv.kvcrush_select(sc, 512, 384, 0, "alternating", 0, unit=16)
    bt = inputs.make_block_table(w, seed)
    kp, vp = inputs.to_paged(k.cuda(), bt, 16), inputs.to_paged(v.cuda(), bt, 16)
    ko, vo = kv.kvcrush_compact(kp, vp, idx, block_table=bt.cuda(), block_size=16, dense_shape=(1, 2, 2048, 128))
    torch.cuda.synchronize()
    ridx, rkind, _ = oracle.select_units(sc.cpu(), 16, 512, 384, 0, "alternating", 0)
    assert torch.equal(idx.cpu(), ridx) and torch.equal(kind.cpu(), rkind)
    rk, rv = oracle.compact(k, v, ridx)
    assert torch.equal(ko.cpu().view(torch.uint8), rk.view(torch.uint8))
    assert torch.equal(vo.cpu().view(torch.uint8), rv.view(torch.uint8))
    # whole blocks are kept: the reduced cache's block table is a gather of the old one, and the
    # pool read through it is the compacted cache (no data was moved)
    pages = idx.cpu()[0, ::16] // 16
    assert torch.equal(idx.cpu()[0].view(-1, 16), (pages[:, None] * 16 + torch.arange(16)[None, :]).to(torch.int32))
    bt_small = kv.kvcrush_compact_block_table(idx, bt.cuda(), 16)
    torch.cuda.synchronize()
    assert torch.equal(bt_small.cpu()[0], bt[0, pages.long()])
    via_table = kp[bt_small[0].long()].permute(2, 0, 1, 3).reshape(2, 512, 128)     # [Hkv, kept tokens, D]
    assert torch.equal(via_table.cpu().view(torch.uint8), rk[0].view(torch.uint8))


def test_per_layer_budgets_share_one_workspace(kv, oracle):
    """A pyramid of budgets over the layers (the PyramidKV pairing): budget and split
    are per-call arguments and the workspace sized for one call serves them all."""
    say("per-layer budgets, one workspace")
    B, Hs, S = 2, 8, 3000
    ws = torch.empty(kv.kvcrush_select_workspace(kv.make_select_args(B, Hs, S, S, S)), dtype=torch.uint8,
                     device="cuda")
    for layer, budget in enumerate([1200, 900, 600, 300, 64]):
        need = kv.kvcrush_select_workspace(kv.make_select_args(B, Hs, S, budget, budget * 3 // 4))
        assert need <= ws.numel()
        sc = inputs.make_scores(B, Hs, S, seed=100 + layer, ties=True)
        idx, kind, _ = kv.kvcrush_select(sc.cuda(), budget, budget * 3 // 4, 0, "mean", layer, workspace=ws)
        torch.cuda.synchronize()
        ridx, rkind, _ = oracle.select(sc, budget, budget * 3 // 4, 0, "mean", layer)
        assert torch.equal(idx.cpu(), ridx) and torch.equal(kind.cpu(), rkind)


@pytest.mark.parametrize("B,Hs,S,budget,n_imp,kbit,anchor,ties", [
    (1, 8, 512, 128, 64, 0, "alternating", False),
    (2, 8, 1000, 300, 225, 0, "mean", True),
    (1, 32, 4096, 1024, 512, 0, "random", False),
    (3, 32, 777, 200, 50, 0, "random", True),
    (1, 1, 64, 16, 8, 0, "alternating", True),
    (1, 33, 65, 20, 5, 0, "mean", True),
    (2, 64, 300, 64, 48, 200, "mean", True),       # kbit > S/2: the mean anchor gets one-bits
    (1, 100, 500, 100, 75, 0, "random", False),    # two bit words per token
    (1, 128, 257, 60, 20, 0, "alternating", True),
    (1, 8, 1, 1, 1, 0, "alternating", False),
    (1, 8, 1, 1, 0, 0, "alternating", False),
    (1, 8, 63, 63, 20, 0, "random", True),         # budget == S: identity
    (2, 8, 200, 50, 0, 0, "alternating", True),    # no important tokens
    (2, 8, 200, 50, 50, 0, "mean", True),          # no representatives
    (1, 8, 200, 0, 0, 7, "mean", False),           # nothing kept
    (1, 8, 16384, 4096, 3072, 0, "mean", False),   # config-3 sizes
    (1, 8, 32768, 1024, 768, 0, "alternating", True),
    (1, 4, 40000, 5000, 3000, 0, "random", True),  # rows too long for LDS: keys go through the workspace
    (8, 8, 8192, 2048, 1536, 0, "alternating", False),
    (200, 4, 150, 40, 20, 0, "random", True),      # many short sequences
    (1, 128, 8192, 1000, 600, 0, "mean", True),    # row bitmaps too large for LDS staging
])
def test_select_matches_oracle(kv, oracle, B, Hs, S, budget, n_imp, kbit, anchor, ties):
    say(f"select B={B} Hs={Hs} S={S} budget={budget} n_imp={n_imp} kbit={kbit} {anchor} ties={ties}")
    sc = inputs.make_scores(B, Hs, S, seed=S * 7 + Hs, ties=ties)
    check_select(kv, oracle, sc, budget, n_imp, kbit, anchor, seed=1234)


def test_select_explicit_anchor_negative_and_zero_scores(kv, oracle):
    say("select explicit anchor, signed scores")
    g = torch.Generator().manual_seed(5)
    sc = torch.randn(2, 70, 333, generator=g)            # negative values, both zero signs
    sc[:, :, ::7] = 0.0
    sc[:, :, 3::11] = -0.0
    ab = torch.randint(-2**62, 2**62, (2, 2), generator=g, dtype=torch.int64)
    check_select(kv, oracle, sc, 100, 40, 0, "explicit", anchor_bits=ab)
    # all scores equal: every decision is a tie
    check_select(kv, oracle, torch.ones(1, 8, 500), 100, 60, 0, "alternating")


def test_select_importance_sum_is_sequential_fp32(kv, oracle):
    """Token importance is the fp32 sum of the score rows in row order; any other order or width
    ranks these three tokens differently ((2 + 1e8) - 1e8 = 0 in fp32)."""
    sc = torch.zeros(1, 3, 4)
    sc[0, :, 0] = torch.tensor([1e8, -1e8, 1.0])
    sc[0, :, 1] = torch.tensor([0.25, 0.25, 0.25])
    sc[0, :, 2] = torch.tensor([2.0, 1e8, -1e8])
    idx, _, _ = kv.kvcrush_select(sc.cuda(), 1, 1, 1, "alternating")
    torch.cuda.synchronize()
    assert idx.cpu().tolist() == [[0]] == oracle.select(sc, 1, 1, 1, "alternating")[0].tolist()
    # the same through the page-level path (units of two tokens: sums 1 + 0.75 and 0 + 0)
    idx2, _, _ = kv.kvcrush_select(sc.cuda(), 2, 2, 1, "alternating", unit=2)
    torch.cuda.synchronize()
    assert idx2.cpu().tolist() == [[0, 1]] == oracle.select_units(sc, 2, 2, 2, 1, "alternating")[0].tolist()


def test_select_is_deterministic(kv):
    sc = inputs.make_scores(2, 8, 5000, seed=3, ties=True).cuda()
    a = kv.kvcrush_select(sc, 1000, 750, want_bits=True)
    b = kv.kvcrush_select(sc, 1000, 750, want_bits=True)
    torch.cuda.synchronize()
    assert all(torch.equal(x, y) for x, y in zip(a, b))


# ------------------------------------------------------------------ stage 1
def check_scores(kv, oracle, w, seed, reduce_groups, check_lse=True):
    q, k, _ = inputs.make_qkv(w, seed, want_v=False)
    sc, ws = kv.kvcrush_scores(q.cuda(), k.cuda(), reduce_groups)
    torch.cuda.synchronize()
    ref, ref_lse = oracle.scores(q, k, reduce_groups, want_lse=True, threads=THREADS)
    err = rel_err(sc, ref)
    assert err <= SCORE_RTOL, f"scores off by {err:.3e} relative"
    if check_lse:
        lse = kv.lse_from_workspace(ws, w.B, w.Hq, w.S).cpu()
        assert (lse.double() - ref_lse.double()).abs().max().item() < 1e-4
    # each head's column sums total the number of query rows
    G = w.Hq // w.Hkv if reduce_groups else 1
    tot = sc.double().sum(-1).cpu()
    assert torch.allclose(tot, torch.full_like(tot, float(G * w.S)), rtol=1e-4)
    # single pass with the caller's lse gives the same result
    sc2, _ = kv.kvcrush_scores(q.cuda(), k.cuda(), reduce_groups, lse=ref_lse.cuda())
    torch.cuda.synchronize()
    assert rel_err(sc2, ref) <= SCORE_RTOL
    # the normalisers on their own, with and without scratch memory for key slices
    if check_lse:
        for ws_arg in ("auto", None):
            lse_alone = kv.kvcrush_row_lse(q.cuda(), k.cuda(), workspace=ws_arg).cpu()
            assert (lse_alone.double() - ref_lse.double()).abs().max().item() < 1e-4
    return sc


@pytest.mark.parametrize("B,Hq,Hkv,S,D,dtype,rg", [
    (1, 8, 8, 512, 64, "f32", False),        # config 1
    (2, 4, 2, 300, 64, "bf16", True),
    (1, 4, 1, 777, 128, "bf16", True),
    (1, 4, 1, 777, 128, "bf16", False),
    (1, 3, 1, 200, 128, "bf16", True),       # odd group size
    (2, 2, 2, 257, 128, "f32", False),
    (1, 2, 1, 129, 64, "f32", True),
    (1, 1, 1, 1, 128, "bf16", False),
    (1, 2, 2, 31, 64, "bf16", False),
    (1, 8, 4, 1024, 128, "bf16", True),
    (1, 4, 2, 2100, 64, "bf16", True),       # several query chunks, D = 64 pipeline
    (1, 2, 2, 1333, 128, "bf16", False),     # several query chunks, ragged tail, one head per row
    (2, 2, 1, 1100, 128, "f32", True),       # fp32 path with partial sums
    (64, 8, 2, 300, 64, "bf16", True),       # many short sequences
    (1, 2, 1, 64, 128, "bf16", True),        # exactly one tile
    (1, 2, 1, 256, 128, "bf16", True),       # exactly one key block
    (1, 2, 1, 1152, 128, "bf16", True),      # exactly one query chunk of pass B
    (1, 2, 1, 1153, 128, "bf16", True),      # one row more
    (1, 2, 1, 2304, 64, "bf16", False),      # exactly two chunks, D = 64
    (1, 8, 2, 1400, 128, "f16", True),       # IEEE half inputs: same tiling, the f16 matrix instruction
    (2, 4, 4, 333, 64, "f16", False),
])
def test_scores_small(kv, oracle, B, Hq, Hkv, S, D, dtype, rg):
    say(f"scores B={B} Hq={Hq} Hkv={Hkv} S={S} D={D} {dtype} reduce_groups={rg}")
    w = inputs.Workload("t", B, Hq, Hkv, S, D, dtype, max(1, S // 4), 0.5, "alternating", rg, sink_bias=True)
    check_scores(kv, oracle, w, seed=S + Hq, reduce_groups=rg)


def test_scores_extreme_logits(kv, oracle):
    """Logits that grow by hundreds along the sequence: the exponentials' fixed
    reference has to be re-based on the fly (and early keys underflow to zero)."""
    say("scores with logits spanning several hundred")
    S, D = 1500, 128
    g = torch.Generator().manual_seed(77)
    q = torch.randn(1, 2, S, D, generator=g)
    k = torch.randn(1, 1, S, D, generator=g)
    ramp = torch.linspace(0.01, 40.0, S)
    ramp[700:] = ramp[700:].flip(0)                      # up, then down again
    k = k * ramp[None, None, :, None]
    q, k = q.to(torch.bfloat16), k.to(torch.bfloat16)
    for rg in (True, False):
        sc, _ = kv.kvcrush_scores(q.cuda(), k.cuda(), rg)
        torch.cuda.synchronize()
        ref = oracle.scores(q, k, rg, threads=THREADS)
        assert torch.isfinite(sc).all()
        # tokens that receive essentially nothing are compared absolutely
        got, want = sc.cpu().double(), ref.double()
        big = want > 1e-30
        assert ((got[big] - want[big]).abs() / want[big]).max().item() <= SCORE_RTOL
        assert got[~big].abs().max().item() <= 1e-30 if (~big).any() else True


@pytest.mark.parametrize("B,Hq,Hkv,S,D,dtype,rg,W", [
    (1, 4, 2, 700, 128, "bf16", True, 32),      # window inside the last tile
    (2, 4, 1, 1000, 128, "bf16", True, 1),      # the last attention row alone
    (1, 2, 2, 900, 64, "bf16", False, 333),     # ragged window start, D = 64
    (1, 4, 2, 4000, 128, "bf16", True, 2500),   # window over several query chunks, tile offset > 0
    (1, 2, 1, 3000, 128, "bf16", True, 1152),   # exactly one chunk of queries
    (1, 2, 2, 1500, 128, "f32", False, 100),    # fp32 path
    (1, 2, 1, 2500, 64, "f32", True, 1300),     # fp32 path, partial sums with a tile offset
    (1, 2, 1, 300, 128, "bf16", True, 300),     # W = S: all rows
    (1, 2, 1, 300, 128, "bf16", True, 5000),    # W > S: all rows
])
def test_scores_observation_window(kv, oracle, B, Hq, Hkv, S, D, dtype, rg, W):
    """Received attention from the last W queries only (the SnapKV baseline's scores)."""
    say(f"window scores B={B} Hq={Hq} Hkv={Hkv} S={S} D={D} {dtype} reduce_groups={rg} W={W}")
    w = inputs.Workload("t", B, Hq, Hkv, S, D, dtype, max(1, S // 4), 0.5, "alternating", rg, sink_bias=True)
    q, k, _ = inputs.make_qkv(w, S + W, want_v=False)
    sc, ws = kv.kvcrush_scores(q.cuda(), k.cuda(), rg, window=W)
    torch.cuda.synchronize()
    ref, ref_lse = oracle.scores(q, k, rg, want_lse=True, threads=THREADS, window=W)
    got, want = sc.cpu().double(), ref.double()
    big = want > 1e-30
    assert ((got[big] - want[big]).abs() / want[big]).max().item() <= SCORE_RTOL
    if (~big).any():
        assert got[~big].abs().max().item() <= 1e-30
    Weff = min(W, S)
    tot = got.sum(-1)
    assert torch.allclose(tot, torch.full_like(tot, float((Hq // Hkv if rg else 1) * Weff)), rtol=1e-4)
    # the normalisers of the window rows are the ones the workspace holds
    lse = kv.lse_from_workspace(ws, B, Hq, S).cpu()
    assert (lse[..., S - Weff:].double() - ref_lse[..., S - Weff:].double()).abs().max().item() < 1e-4
    # a caller-supplied lse is read inside the window only: garbage before it is harmless
    junk = ref_lse.clone()
    junk[..., : S - Weff] = float("nan")
    sc2, _ = kv.kvcrush_scores(q.cuda(), k.cuda(), rg, lse=junk.cuda(), window=W)
    torch.cuda.synchronize()
    got2 = sc2.cpu().double()
    assert torch.isfinite(got2).all()
    assert ((got2[big] - want[big]).abs() / want[big]).max().item() <= SCORE_RTOL
    # row_lse on its own writes the same window rows
    lse2 = kv.kvcrush_row_lse(q.cuda(), k.cuda(), window=W).cpu()
    assert torch.equal(lse2[..., S - Weff:], lse[..., S - Weff:])
    # ... and without scratch memory (keys not cut into slices) agrees to rounding
    lse3 = kv.kvcrush_row_lse(q.cuda(), k.cuda(), window=W, workspace=None).cpu()
    assert (lse3[..., S - Weff:].double() - ref_lse[..., S - Weff:].double()).abs().max().item() < 1e-4


@pytest.mark.parametrize("rows,S,kernel", [((2, 3), 37, 1), ((1, 8), 1000, 7), ((3,), 2048, 5), ((2, 2), 2049, 13),
                                           ((1,), 5000, 1023), ((4,), 6, 41), ((1, 1), 1, 3), ((8, 8), 16384, 7)])
def test_pool_scores(kv, oracle, rows, S, kernel):
    say(f"max pool rows={rows} S={S} kernel={kernel}")
    x = torch.randn(*rows, S, generator=torch.Generator().manual_seed(S + kernel))
    x = (x * 4).round() / 4  # plenty of equal values
    got = kv.kvcrush_pool_scores(x.cuda(), kernel)
    torch.cuda.synchronize()
    assert torch.equal(got.cpu(), oracle.maxpool(x, kernel))


def test_pool_scores_rejects_bad_arguments(kv):
    x = torch.zeros(2, 64, device="cuda")
    for kernel in (0, 2, 1025, -3):
        with pytest.raises(kv.KVCrushError):
            kv.kvcrush_pool_scores(x, kernel)
    with pytest.raises(kv.KVCrushError):
        kv.kvcrush_pool_scores(x, 3, out=x)                   # in place is not supported
    with pytest.raises(kv.KVCrushError):
        kv.kvcrush_pool_scores(x.view(-1)[:64].view(1, 64), 3, out=x.view(-1)[32:96].view(1, 64))


def test_window_pool_topk_pipeline(kv, oracle):
    """The SnapKV-style baseline end to end: window scores, pooling, plain top-k
    (budget == n_important, so no representatives), gather."""
    say("window -> pool -> top-k -> gather")
    w = inputs.Workload("t", 2, 8, 2, 2000, 128, "bf16", 500, 1.0, "alternating", True, sink_bias=True)
    q, k, v = inputs.make_qkv(w, 5)
    sc, _ = kv.kvcrush_scores(q.cuda(), k.cuda(), True, window=64)
    pooled = kv.kvcrush_pool_scores(sc, 7)
    idx, kind, _ = kv.kvcrush_select(pooled, 500, 500)
    ko, vo = kv.kvcrush_compact(k.cuda(), v.cuda(), idx)
    torch.cuda.synchronize()
    ref_pooled = oracle.maxpool(sc.cpu(), 7)
    assert torch.equal(pooled.cpu(), ref_pooled)
    ridx, rkind, _ = oracle.select(ref_pooled, 500, 500)
    assert torch.equal(idx.cpu(), ridx) and torch.equal(kind.cpu(), rkind)
    rk, rv = oracle.compact(k, v, ridx)
    assert torch.equal(ko.cpu().view(torch.uint8), rk.view(torch.uint8))
    assert torch.equal(vo.cpu().view(torch.uint8), rv.view(torch.uint8))


@pytest.mark.parametrize("Dtrue,Dpad,S,W", [(96, 128, 1100, 0), (96, 128, 700, 64), (40, 64, 500, 0)])
def test_scores_padded_heads_with_their_own_scale(kv, oracle, Dtrue, Dpad, S, W):
    """Heads of 96 values (Phi-3-mini among the paper's models) or 40: zero-padded to the next
    supported size and scored with 1/sqrt(true size); the oracle works on the unpadded heads."""
    say(f"scores with D={Dtrue} padded to {Dpad}, softmax_scale=1/sqrt({Dtrue}), S={S} window={W}")
    g = torch.Generator().manual_seed(Dtrue + S)
    q = torch.randn(2, 4, S, Dtrue, generator=g).to(torch.bfloat16)
    k = torch.randn(2, 2, S, Dtrue, generator=g).to(torch.bfloat16)
    pad = lambda t: torch.cat([t, torch.zeros(*t.shape[:-1], Dpad - Dtrue, dtype=t.dtype)], dim=-1).contiguous()
    scale = 1.0 / (Dtrue ** 0.5)
    sc, _ = kv.kvcrush_scores(pad(q).cuda(), pad(k).cuda(), True, window=W, scale=scale)
    torch.cuda.synchronize()
    ref = oracle.scores(q, k, True, threads=THREADS, window=W)
    got, want = sc.cpu().double(), ref.double()
    big = want > 1e-30
    assert ((got[big] - want[big]).abs() / want[big]).max().item() <= SCORE_RTOL
    # the decoding step takes the same scale
    old = torch.rand(2, 2, S, generator=g)
    app = kv.kvcrush_scores_append(pad(q)[:, :, -1].contiguous().cuda(), pad(k).cuda(), old.clone().cuda(), S, True,
                                   scale=scale)
    torch.cuda.synchronize()
    assert rel_err(app, oracle.scores_append(q[:, :, -1].contiguous(), k, old.clone(), S, True)) <= SCORE_RTOL


def test_scores_deterministic(kv):
    w = inputs.Workload("t", 1, 8, 2, 1500, 128, "bf16", 256, 0.5, "alternating", True)
    q, k, _ = inputs.make_qkv(w, 1, want_v=False)
    a, _ = kv.kvcrush_scores(q.cuda(), k.cuda(), True)
    b, _ = kv.kvcrush_scores(q.cuda(), k.cuda(), True)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


# -------------------------------------------------------- whole path, configs
def run_pipeline(kv, oracle, w, cfg_id, layer, check_groups, whole=False):
    """GPU runs the full configuration; the oracle checks the score rows in
    `check_groups` (list of (b, row); whole=True: every row, in one oracle call that
    keeps all host cores busy) plus the whole selection and compaction, the latter
    two on the GPU's own score tensor."""
    seed = inputs.layer_seed(cfg_id, layer)
    q, k, v = inputs.make_qkv(w, seed)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    sc, ws = kv.kvcrush_scores(qd, kd, w.reduce_groups)
    idx, kind, bits = kv.kvcrush_select(sc, w.budget, w.n_important, 0, w.anchor, inputs.anchor_seed(layer),
                                        want_bits=True)
    if w.paged:
        bt = inputs.make_block_table(w, seed)
        kp, vp = inputs.to_paged(kd, bt, w.block_size), inputs.to_paged(vd, bt, w.block_size)
        ko, vo = kv.kvcrush_compact(kp, vp, idx, block_table=bt.cuda(), block_size=w.block_size,
                                    dense_shape=(w.B, w.Hkv, w.S, w.D))
    else:
        ko, vo = kv.kvcrush_compact(kd, vd, idx)
    torch.cuda.synchronize()
    sc_h = sc.cpu()
    G = w.Hq // w.Hkv
    # stage 1: rows against the oracle, invariant on all rows
    if whole:
        ref = oracle.scores(q, k, w.reduce_groups, threads=THREADS)
        err = rel_err(sc_h, ref)
        say(f"  cfg{cfg_id} layer {layer}: score rel err over all {w.B * w.Hs} rows {err:.3e}")
        assert err <= SCORE_RTOL
        check_groups = []
    elif isinstance(check_groups, range):
        # consecutive KV groups of every sequence in one oracle call (reduce_groups workloads)
        r0, r1 = check_groups.start, check_groups.stop
        ref = oracle.scores(q[:, r0 * G:r1 * G].contiguous(), k[:, r0:r1].contiguous(), True, threads=THREADS)
        err = rel_err(sc_h[:, r0:r1], ref)
        say(f"  cfg{cfg_id} layer {layer}: score rel err over rows {r0}..{r1 - 1} {err:.3e}")
        assert err <= SCORE_RTOL
        check_groups = []
    for (b, row) in check_groups:
        if w.reduce_groups:
            ref = oracle.scores(q[b:b + 1, row * G:(row + 1) * G], k[b:b + 1, row:row + 1], True, threads=THREADS)
        else:
            ref = oracle.scores(q[b:b + 1, row:row + 1], k[b:b + 1, row // G:row // G + 1], False)
        err = rel_err(sc_h[b, row], ref[0, 0])
        say(f"  cfg{cfg_id} layer {layer} (b={b}, row={row}): score rel err {err:.3e}")
        assert err <= SCORE_RTOL
    tot = sc_h.double().sum(-1)
    per_row = float((G if w.reduce_groups else 1) * w.S)
    assert torch.allclose(tot, torch.full_like(tot, per_row), rtol=1e-4)
    assert (sc_h > 0).all()
    # stages 2-4 on the GPU's scores: bit-exact
    ridx, rkind, rbits = oracle.select(sc_h, w.budget, w.n_important, 0, w.anchor, inputs.anchor_seed(layer))
    assert torch.equal(bits.cpu(), rbits)
    assert torch.equal(idx.cpu(), ridx)
    assert torch.equal(kind.cpu(), rkind)
    # stage 5: bit-exact rows (dense oracle gather on the original tensors)
    rk, rv = oracle.compact(k, v, ridx)
    assert torch.equal(ko.cpu().view(torch.uint8), rk.view(torch.uint8))
    assert torch.equal(vo.cpu().view(torch.uint8), rv.view(torch.uint8))


def test_config1_full(kv, oracle):
    say("config 1: all heads")
    w = inputs.CONFIGS[1]
    run_pipeline(kv, oracle, w, 1, 0, [(0, r) for r in range(w.Hs)])


def test_config2_full(kv, oracle):
    say("config 2: all 32 heads against the oracle")
    w = inputs.CONFIGS[2]
    q, k, _ = inputs.make_qkv(w, inputs.layer_seed(2, 0), want_v=False)
    sc, _ = kv.kvcrush_scores(q.cuda(), k.cuda(), False)
    torch.cuda.synchronize()
    ref = oracle.scores(q, k, False, threads=THREADS)
    err = rel_err(sc, ref)
    say(f"  cfg2 score rel err {err:.3e}")
    assert err <= SCORE_RTOL
    run_pipeline(kv, oracle, w, 2, 0, [])


def all_rows(w):
    return [(b, r) for b in range(w.B) for r in range(w.Hs)]


@pytest.mark.slow
@pytest.mark.parametrize("layer", [0, 15, 31])
def test_config3_layers(kv, oracle, layer):
    say(f"config 3 layer {layer}: every score row against the oracle, selection and gather in full")
    w = inputs.CONFIGS[3]
    run_pipeline(kv, oracle, w, 3, layer, all_rows(w), whole=True)


@pytest.mark.slow
def test_config4_batched(kv, oracle):
    say("config 4: B=8, every (sequence, group) row against the oracle")
    w = inputs.CONFIGS[4]
    run_pipeline(kv, oracle, w, 4, 0, all_rows(w), whole=True)


@pytest.mark.slow
@pytest.mark.parametrize("layer,rows", [(0, range(0, 4)), (0, range(4, 8)), (15, [3]), (31, [6])])
def test_config5_long_paged(kv, oracle, layer, rows):
    """Every score row of layer 0 (in two halves, so that no single test holds the host's cores for
    long), one row each of layers 15 and 31."""
    say(f"config 5 layer {layer}: S=32768, paged gather, score rows {list(rows)} against the oracle")
    w = inputs.CONFIGS[5]
    run_pipeline(kv, oracle, w, 5, layer, rows if isinstance(rows, range) else [(0, r) for r in rows])


@pytest.mark.slow
def test_config3_one_bit_per_query_head(kv, oracle):
    """Sec. 4.3.3 counts 32 bits per token for a Llama-3-8B layer: one bit per QUERY head.  The
    config-3 layer with reduce_groups = 0 (32 score rows of 16384 tokens under grouped-query
    attention): every row against the oracle, then selection on the 32-bit vectors and the
    gather, bit-exact, in the launch shapes the benchmark's per-head variant times."""
    import dataclasses
    say("config 3 shape, one score row per query head: 32 rows against the oracle, selection and gather")
    w = dataclasses.replace(inputs.CONFIGS[3], name="cfg3_per_query_head_bits", reduce_groups=False)
    assert w.Hs == 32
    run_pipeline(kv, oracle, w, 3, 0, all_rows(w), whole=True)


LAYER_GROUPS = [range(g, g + 4) for g in range(0, 32, 4)]


@pytest.mark.slow
@pytest.mark.parametrize("cfg_id", [3, 5])
@pytest.mark.parametrize("layers", LAYER_GROUPS, ids=lambda r: f"layers{r.start}-{r.stop - 1}")
def test_every_layer_of_the_32_layer_configs(kv, oracle, cfg_id, layers):
    """Configs 3 and 5 are 32 layers with seeds of their own.  On every layer: each score row
    totals the number of query rows it sums (times the group size) and is positive; selection and
    gather (paged for config 5) on the GPU's own scores are bit-exact against the oracle.  (The
    oracle's score pass, minutes per layer, runs on layers 0, 15 and 31 in the tests above.)"""
    w = inputs.CONFIGS[cfg_id]
    for layer in layers:
        say(f"config {cfg_id} layer {layer}: row totals, selection and gather")
        run_pipeline(kv, oracle, w, cfg_id, layer, [])


# ------------------------------------------------------------------ decoding
@pytest.mark.parametrize("B,Hq,Hkv,S,cap,D,dtype,rg", [
    (2, 8, 2, 300, 320, 128, "bf16", True),
    (1, 4, 4, 257, 257, 64, "bf16", False),       # ragged: one key in the last block, capacity == S
    (3, 4, 1, 1, 16, 128, "bf16", True),          # the very first token
    (1, 12, 1, 700, 1024, 128, "bf16", True),     # 12 heads share one KV head: two register chunks
    (2, 2, 2, 513, 600, 128, "f32", False),
    (1, 6, 3, 100, 128, 64, "f32", True),
    (8, 32, 8, 2049, 2304, 128, "bf16", True),    # a compressed config-4 cache in mid-generation
    (2, 8, 2, 777, 800, 128, "f16", True),
])
def test_scores_append_matches_oracle(kv, oracle, B, Hq, Hkv, S, cap, D, dtype, rg):
    say(f"append B={B} Hq={Hq} Hkv={Hkv} S={S} capacity={cap} D={D} {dtype} reduce_groups={rg}")
    td = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[dtype]
    g = torch.Generator().manual_seed(S + Hq)
    qn = torch.randn(B, Hq, D, generator=g).to(td)
    kc = torch.randn(B, Hkv, cap, D, generator=g).to(td)
    kc[:, :, :4] *= 2.0                                    # a few strongly attended early tokens
    Hs = Hkv if rg else Hq
    old = torch.rand(B, Hs, cap, generator=g) * 3.0
    got = kv.kvcrush_scores_append(qn.cuda(), kc.cuda(), old.clone().cuda(), S, rg)
    torch.cuda.synchronize()
    want = oracle.scores_append(qn, kc, old.clone(), S, rg)
    assert torch.equal(got.cpu()[:, :, S:], old[:, :, S:]), "entries beyond the valid length were touched"
    assert rel_err(got[:, :, :S], want[:, :, :S]) <= SCORE_RTOL
    # what was added is one probability row per head
    added = got.cpu().double()[:, :, :S].sum(-1) - old.double()[:, :, :S - 1].sum(-1)
    assert torch.allclose(added, torch.full_like(added, float(Hq // Hkv if rg else 1)), rtol=1e-4)


def test_prefix_plus_appends_equals_prefill(kv):
    """Identity across the two score paths of the library itself: prefill scores of a prefix plus
    one append per later token equal the prefill scores of the whole sequence."""
    say("prefill(S0) + appends == prefill(S)")
    w = inputs.Workload("t", 2, 8, 2, 400, 128, "bf16", 100, 0.5, "alternating", True, sink_bias=True)
    q, k, _ = inputs.make_qkv(w, 3, want_v=False)
    qd, kd = q.cuda(), k.cuda()
    S0, S, cap = 330, 400, 448
    whole, _ = kv.kvcrush_scores(qd, kd, True)
    sc = torch.zeros(2, 2, cap, device="cuda")
    sc[:, :, :S0] = kv.kvcrush_scores(qd[:, :, :S0].contiguous(), kd[:, :, :S0].contiguous(), True)[0]
    kc = torch.zeros(2, 2, cap, 128, dtype=torch.bfloat16, device="cuda")
    kc[:, :, :S] = kd
    for n in range(S0 + 1, S + 1):
        kv.kvcrush_scores_append(qd[:, :, n - 1].contiguous(), kc, sc, n, True)
    torch.cuda.synchronize()
    assert rel_err(sc[:, :, :S], whole.cpu()) <= 1e-4


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_compact_cache_matches_oracle(kv, oracle, dtype):
    say(f"eviction gather on capacity-strided caches, {dtype}")
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    B, Hkv, Hs, D, cap_src, cap_dst, budget = 3, 4, 4, 128, 700, 520, 333
    g = torch.Generator().manual_seed(8)
    k = torch.randn(B, Hkv, cap_src, D, generator=g).to(td)
    v = torch.randn(B, Hkv, cap_src, D, generator=g).to(td)
    sc = torch.randn(B, Hs, cap_src, generator=g)
    idx = torch.stack([torch.randperm(650, generator=g)[:budget].sort().values for _ in range(B)]).to(torch.int32)
    outs = [torch.full((B, Hkv, cap_dst, D), 5.0, dtype=td), torch.full((B, Hkv, cap_dst, D), 6.0, dtype=td),
            torch.full((B, Hs, cap_dst), 7.0)]
    want = oracle.compact_cache(k, v, sc, idx, *[t.clone() for t in outs])
    got = kv.kvcrush_compact_cache(k.cuda(), v.cuda(), sc.cuda(), idx.cuda(), *[t.clone().cuda() for t in outs])
    torch.cuda.synchronize()
    for a, b in zip(got, want):
        assert torch.equal(a.cpu().view(torch.uint8), b.view(torch.uint8))


def test_decode_loop_with_evictions(kv, oracle):
    """Generation loop: compress after prefill (protected ends), then append token by token and
    evict whenever the cache is full.  The oracle replays every step on its own state; each
    eviction is compared on the GPU's own score tensor (bit-exact) and applied to both sides."""
    say("decode loop: prefill -> compress -> 150 x append, eviction whenever the cache is full")
    B, Hq, Hkv, D, S0 = 2, 8, 2, 128, 600
    budget, n_imp, sink, recent, cap, steps = 200, 90, 8, 32, 256, 150
    w = inputs.Workload("t", B, Hq, Hkv, S0 + steps, D, "bf16", budget, 0.5, "alternating", True, sink_bias=True)
    q, k, v = inputs.make_qkv(w, 17)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()

    def evict(sc_dev, valid, kc, vc, o_state):
        idx, kind, _ = kv.kvcrush_select(sc_dev, budget, n_imp, 0, "mean", 3, n_sink=sink, n_recent=recent,
                                         valid_len=valid)
        torch.cuda.synchronize()
        ridx, rkind, _ = oracle.select(sc_dev.cpu()[:, :, :valid].contiguous(), budget, n_imp, 0, "mean", 3,
                                       n_sink=sink, n_recent=recent)
        assert torch.equal(idx.cpu(), ridx) and torch.equal(kind.cpu(), rkind)
        new = [torch.zeros_like(kc), torch.zeros_like(vc), torch.zeros_like(sc_dev)]
        kv.kvcrush_compact_cache(kc, vc, sc_dev, idx, *new)
        o_new = [torch.zeros_like(t) for t in o_state]
        oracle.compact_cache(*o_state, ridx, *o_new)
        return new, o_new

    # prefill + first compression (dense tensors: capacity == S0)
    sc0, _ = kv.kvcrush_scores(qd[:, :, :S0].contiguous(), kd[:, :, :S0].contiguous(), True)
    o_sc0 = oracle.scores(q[:, :, :S0].contiguous(), k[:, :, :S0].contiguous(), True, threads=THREADS)
    assert rel_err(sc0, o_sc0) <= SCORE_RTOL
    pad = lambda t, n: torch.cat([t, torch.zeros(*t.shape[:2], n - t.shape[2], *t.shape[3:], dtype=t.dtype,
                                                 device=t.device)], dim=2)
    (kc, vc, sc), (o_k, o_v, o_sc) = evict(pad(sc0, S0), S0, kd[:, :, :S0].contiguous(), vd[:, :, :S0].contiguous(),
                                           [k[:, :, :S0].contiguous(), v[:, :, :S0].contiguous(), o_sc0])
    # move into capacity-sized caches
    kc, vc, sc = [t[:, :, :cap].contiguous() for t in (kc, vc, sc)]
    o_k, o_v, o_sc = [t[:, :, :cap].contiguous() for t in (o_k, o_v, o_sc)]
    n, evictions = budget, 0
    for step in range(steps):
        pos = S0 + step
        if n == cap:
            (kc, vc, sc), (o_k, o_v, o_sc) = evict(sc, n, kc, vc, [o_k, o_v, o_sc])
            n, evictions = budget, evictions + 1
        kc[:, :, n] = kd[:, :, pos]
        vc[:, :, n] = vd[:, :, pos]
        o_k[:, :, n] = k[:, :, pos]
        o_v[:, :, n] = v[:, :, pos]
        n += 1
        kv.kvcrush_scores_append(qd[:, :, pos].contiguous(), kc, sc, n, True)
        oracle.scores_append(q[:, :, pos].contiguous(), o_k, o_sc, n, True)
    torch.cuda.synchronize()
    assert evictions == 2
    assert torch.equal(kc.cpu()[:, :, :n].view(torch.uint8), o_k[:, :, :n].view(torch.uint8))
    assert torch.equal(vc.cpu()[:, :, :n].view(torch.uint8), o_v[:, :, :n].view(torch.uint8))
    assert rel_err(sc[:, :, :n], o_sc[:, :, :n]) <= SCORE_RTOL


# ------------------------------------------------------------------ HIP graphs
def test_whole_path_replays_from_a_hip_graph(kv, oracle):
    """The entry points only enqueue kernels on the caller's stream and allocate nothing, so a
    layer's compression can be captured once and replayed.  Three replays on fresh inputs, eager
    work and synchronisations in between, each compared with the eager result and the oracle."""
    say("graph capture of scores -> select -> compact, three replays")
    w = inputs.Workload("t", 2, 8, 2, 1500, 128, "bf16", 400, 0.25, "mean", True, sink_bias=True)
    dev = torch.device("cuda")
    q = torch.empty(w.B, w.Hq, w.S, w.D, dtype=torch.bfloat16, device=dev)
    k = torch.empty(w.B, w.Hkv, w.S, w.D, dtype=torch.bfloat16, device=dev)
    v = torch.empty_like(k)
    shape = kv.make_shape(q, k, True)
    ws = torch.empty(kv.kvcrush_scores_workspace(shape), dtype=torch.uint8, device=dev)
    sel_ws = torch.empty(kv.kvcrush_select_workspace(kv.make_select_args(w.B, w.Hkv, w.S, 400, 300, n_sink=4,
                                                                        n_recent=16)), dtype=torch.uint8, device=dev)
    sc = torch.empty(w.B, w.Hkv, w.S, device=dev)
    idx = torch.empty(w.B, 400, dtype=torch.int32, device=dev)
    ko = torch.empty(w.B, w.Hkv, 400, w.D, dtype=torch.bfloat16, device=dev)
    vo = torch.empty_like(ko)

    def layer():
        kv.kvcrush_scores(q, k, True, scores=sc, workspace=ws)
        kv.kvcrush_select(sc, 400, 300, 0, "mean", 5, want_kind=False, idx=idx, workspace=sel_ws, n_sink=4,
                          n_recent=16)
        kv.kvcrush_compact(k, v, idx, k_out=ko, v_out=vo, validate=False)

    def load(seed):
        a, b, c = inputs.make_qkv(w, seed)
        q.copy_(a); k.copy_(b); v.copy_(c)
        return a, b, c

    load(100)
    layer()                                   # eager warm-up (also sets kernel attributes)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            layer()
    torch.cuda.synchronize()
    for seed in (101, 102, 103):
        hq, hk, hv = load(seed)
        ko.zero_(); vo.zero_(); idx.zero_(); sc.zero_()
        g.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (sc, idx, ko, vo)]
        layer()                               # the same work eagerly, on the same inputs
        torch.cuda.synchronize()
        for a, b in zip(got, (sc, idx, ko, vo)):
            assert torch.equal(a, b), "graph replay differs from the eager run"
        ridx, _, _ = oracle.select(got[0].cpu(), 400, 300, 0, "mean", 5, n_sink=4, n_recent=16)
        assert torch.equal(got[1].cpu(), ridx)
        rk, rv = oracle.compact(hk, hv, ridx)
        assert torch.equal(got[2].cpu().view(torch.uint8), rk.view(torch.uint8))
    ref = oracle.scores(hq, hk, True, threads=THREADS)
    assert rel_err(got[0], ref) <= SCORE_RTOL


def test_decode_steps_replay_from_a_hip_graph(kv, oracle):
    say("graph capture of a decoding step, replays at growing cache lengths need one graph per length")
    B, Hq, Hkv, D, cap = 2, 8, 2, 128, 512
    dev = torch.device("cuda")
    g0 = torch.Generator().manual_seed(9)
    kc_h = torch.randn(B, Hkv, cap, D, generator=g0).to(torch.bfloat16)
    kc, sc = kc_h.cuda(), torch.zeros(B, Hkv, cap, device=dev)
    qn = torch.empty(B, Hq, D, dtype=torch.bfloat16, device=dev)
    ws = torch.empty(kv.kvcrush_scores_append_workspace(kv.Shape(B, Hq, Hkv, cap, D, kv.BF16, 1, 0), cap),
                     dtype=torch.uint8, device=dev)
    o_sc = torch.zeros(B, Hkv, cap)
    side = torch.cuda.Stream()
    for n in (300, 301, 302):
        q_h = torch.randn(B, Hq, D, generator=g0).to(torch.bfloat16)
        qn.copy_(q_h)
        kv.kvcrush_scores_append(qn, kc, sc.clone(), n, True, workspace=ws)     # eager warm-up on a copy
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()                  # the cache length is a launch argument: one graph per step
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                kv.kvcrush_scores_append(qn, kc, sc, n, True, workspace=ws)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        oracle.scores_append(q_h, kc_h, o_sc, n, True)
        assert rel_err(sc[:, :, :n], o_sc[:, :, :n]) <= SCORE_RTOL


def test_decode_with_device_lengths_one_graph_for_all_steps(kv, oracle):
    """Sequences of different lengths, the lengths living on the device: one captured launch
    sequence serves every decoding step (the host only bumps the length tensor)."""
    say("decode append with per-sequence device lengths, one graph replayed over 5 steps")
    B, Hq, Hkv, D, cap = 3, 8, 2, 128, 640
    dev = torch.device("cuda")
    g0 = torch.Generator().manual_seed(12)
    kc_h = torch.randn(B, Hkv, cap, D, generator=g0).to(torch.bfloat16)
    start = [37, 300, 513]                                   # one, two and three key blocks
    lens = torch.tensor(start, dtype=torch.int32, device=dev)
    sc_h = torch.rand(B, Hkv, cap, generator=g0)
    kc, sc = kc_h.cuda(), sc_h.clone().cuda()
    qn = torch.zeros(B, Hq, D, dtype=torch.bfloat16, device=dev)
    bound = 600                                              # upper bound that sizes launch and workspace
    ws = torch.empty(kv.kvcrush_scores_append_workspace(kv.Shape(B, Hq, Hkv, bound, D, kv.BF16, 1, 0), cap),
                     dtype=torch.uint8, device=dev)
    scratch = sc.clone()
    kv.kvcrush_scores_append(qn, kc, scratch, bound, True, workspace=ws, lengths=lens)   # eager warm-up
    torch.cuda.synchronize()
    graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            kv.kvcrush_scores_append(qn, kc, sc, bound, True, workspace=ws, lengths=lens)
    torch.cuda.synchronize()
    o_sc = sc_h.clone()
    for step in range(5):
        q_h = torch.randn(B, Hq, D, generator=g0).to(torch.bfloat16)
        qn.copy_(q_h)
        lens.add_(1)                                         # every sequence got one more token
        graph.replay()
        torch.cuda.synchronize()
        for b in range(B):                                   # the oracle takes one length per call
            n = start[b] + step + 1
            part = o_sc[b:b + 1].clone()
            oracle.scores_append(q_h[b:b + 1], kc_h[b:b + 1], part, n, True)
            o_sc[b] = part[0]
            assert rel_err(sc[b, :, :n], o_sc[b, :, :n]) <= SCORE_RTOL, (step, b)
            assert torch.equal(sc[b, :, n:].cpu(), sc_h[b, :, n:]), "entries beyond a sequence's length were touched"


def test_scores_long_sequence_index_arithmetic(kv, oracle):
    """S = 100000 (ragged, 391 key blocks, 87 query chunks): the oracle can afford the last 64
    query rows, which fix the window scores everywhere and the full scores of the last 64 tokens
    (only those rows reach them); the full scores also get the row-total invariant."""
    say("scores at S=100000: window W=64 against the oracle, full scores' tail and totals")
    w = inputs.Workload("t", 1, 4, 1, 100000, 128, "bf16", 1000, 0.25, "alternating", True, sink_bias=True)
    q, k, _ = inputs.make_qkv(w, 4, want_v=False)
    qd, kd = q.cuda(), k.cuda()
    win, _ = kv.kvcrush_scores(qd, kd, True, window=64)
    full, _ = kv.kvcrush_scores(qd, kd, True)
    torch.cuda.synchronize()
    ref = oracle.scores(q, k, True, threads=THREADS, window=64)
    got, want = win.cpu().double(), ref.double()
    big = want > 1e-30
    assert ((got[big] - want[big]).abs() / want[big]).max().item() <= SCORE_RTOL
    assert rel_err(full[..., -64:], ref[..., -64:]) <= SCORE_RTOL
    tot = full.double().sum(-1).cpu()
    assert torch.allclose(tot, torch.full_like(tot, 4.0 * w.S), rtol=1e-4)
    assert (full > 0).all()


def test_select_random_sweep(kv, oracle):
    """Seeded sweep over shapes, budgets, anchors, protected ends and unit sizes (60 cases)."""
    import random
    rng = random.Random(20250300)
    for case in range(60):
        unit = rng.choice([1, 1, 1, 2, 4, 8, 16, 32])
        Hs = rng.choice([1, 2, 3, 8, 8, 17, 32, 64, 100])
        while Hs * unit > 1024:
            Hs //= 2
        B = rng.choice([1, 1, 2, 3])
        n_units = rng.randint(1, 6000 // unit) if rng.random() < 0.8 else rng.randint(1, 20)
        sink = rng.choice([0, 0, 0, 1, 4, 32, 70])
        recent = rng.choice([0, 0, 0, 1, 16, 128])
        Sm = n_units * unit
        S = Sm + sink + recent
        bu = rng.randint(0, n_units)                      # kept units
        iu = rng.randint(0, bu)                           # of which important
        if rng.random() < 0.15:
            iu = bu
        if rng.random() < 0.1:
            iu = 0
        budget, n_imp = bu * unit + sink + recent, iu * unit
        kbit = rng.choice([0, 0, rng.randint(0, Sm)])
        anchor = rng.choice(["alternating", "mean", "random"])
        ties = rng.random() < 0.6
        say(f"  sweep {case}: B={B} Hs={Hs} S={S} unit={unit} budget={budget} n_imp={n_imp} kbit={kbit} "
            f"sink={sink} recent={recent} {anchor} ties={ties}")
        sc = inputs.make_scores(B, Hs, S, seed=1000 + case, ties=ties)
        kw = dict(n_sink=sink, n_recent=recent)
        idx, kind, _ = kv.kvcrush_select(sc.cuda(), budget, n_imp, kbit, anchor, case, unit=unit, **kw)
        torch.cuda.synchronize()
        if unit > 1:
            ridx, rkind, _ = oracle.select_units(sc, unit, budget, n_imp, kbit, anchor, case, **kw)
        else:
            ridx, rkind, _ = oracle.select(sc, budget, n_imp, kbit, anchor, case, **kw)
        assert torch.equal(idx.cpu(), ridx) and torch.equal(kind.cpu(), rkind), f"case {case}"


def test_scores_random_sweep(kv, oracle):
    """Seeded sweep over small score shapes: dtype, head dim, grouping, window, ragged lengths."""
    import random
    rng = random.Random(77)
    for case in range(24):
        dtype = rng.choice(["bf16", "bf16", "f32"])
        D = rng.choice([64, 128])
        Hkv = rng.choice([1, 2, 3])
        G = rng.choice([1, 2, 3, 4, 8])
        B = rng.choice([1, 2])
        S = rng.choice([rng.randint(1, 300), rng.randint(300, 1500), rng.randint(1500, 2600)])
        if dtype == "f32":
            S = min(S, 900)
        rg = rng.random() < 0.6
        W = rng.choice([0, 0, 1, rng.randint(1, S), S + 5])
        say(f"  sweep {case}: B={B} Hq={Hkv * G} Hkv={Hkv} S={S} D={D} {dtype} reduce_groups={rg} window={W}")
        w = inputs.Workload("t", B, Hkv * G, Hkv, S, D, dtype, max(1, S // 4), 0.5, "alternating", rg, sink_bias=True)
        q, k, _ = inputs.make_qkv(w, 500 + case, want_v=False)
        sc, _ = kv.kvcrush_scores(q.cuda(), k.cuda(), rg, window=W)
        torch.cuda.synchronize()
        ref = oracle.scores(q, k, rg, threads=THREADS, window=W)
        got, want = sc.cpu().double(), ref.double()
        big = want > 1e-30
        assert ((got[big] - want[big]).abs() / want[big]).max().item() <= SCORE_RTOL, f"case {case}"
        if (~big).any():
            assert got[~big].abs().max().item() <= 1e-30


@pytest.mark.parametrize("B,Hq,Hkv,S,cap,D,dtype,rg,bs", [
    (2, 8, 2, 300, 320, 128, "bf16", True, 16),
    (1, 4, 4, 257, 288, 64, "bf16", False, 32),
    (2, 2, 2, 513, 640, 128, "f32", False, 16),
    (8, 32, 8, 2049, 2304, 128, "bf16", True, 16),
])
def test_scores_append_on_a_paged_pool(kv, oracle, B, Hq, Hkv, S, cap, D, dtype, rg, bs):
    """The K cache lives in a pool of blocks scattered by a random block table; the oracle reads
    the same keys from the dense tensor they were scattered from."""
    say(f"paged append B={B} Hq={Hq} Hkv={Hkv} S={S} capacity={cap} D={D} {dtype} block={bs}")
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    g = torch.Generator().manual_seed(S + bs)
    qn = torch.randn(B, Hq, D, generator=g).to(td)
    kc = torch.randn(B, Hkv, cap, D, generator=g).to(td)
    nb = cap // bs
    bt = torch.randperm(B * nb, generator=g).to(torch.int32).view(B, nb)
    pool = inputs.to_paged(kc, bt, bs)
    Hs = Hkv if rg else Hq
    old = torch.rand(B, Hs, cap, generator=g)
    got = kv.kvcrush_scores_append(qn.cuda(), pool.cuda(), old.clone().cuda(), S, rg, block_table=bt.cuda(),
                                   block_size=bs)
    dense = kv.kvcrush_scores_append(qn.cuda(), kc.cuda(), old.clone().cuda(), S, rg)
    torch.cuda.synchronize()
    want = oracle.scores_append(qn, kc, old.clone(), S, rg)
    assert rel_err(got[:, :, :S], want[:, :, :S]) <= SCORE_RTOL
    assert torch.equal(got.cpu()[:, :, S:], old[:, :, S:])
    assert torch.equal(got, dense), "paged and dense caches must give identical bits"


# ------------------------------------------------------------------ pipeline classes
def test_layer_compressor_and_decode_cache(kv, oracle):
    """The buffer-owning wrappers (marshalling only): a layer compressed eagerly and from a captured
    graph, then a decoding cache fed token by token; every step replayed by the oracle."""
    say("LayerCompressor (eager + graph) and DecodeCache against the oracle")
    from paper_2503_00022_amd import pipeline
    B, Hq, Hkv, D, S0, steps = 2, 8, 2, 128, 900, 70
    budget, n_imp, sink, recent, cap = 256, 160, 4, 32, 288
    w = inputs.Workload("t", B, Hq, Hkv, S0 + steps, D, "bf16", budget, 0.5, "mean", True, sink_bias=True)
    q, k, v = inputs.make_qkv(w, 23)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    q0, k0, v0 = [t[:, :, :S0].contiguous() for t in (qd, kd, vd)]
    lc = pipeline.LayerCompressor(B, Hq, Hkv, S0, D, torch.bfloat16, budget, n_imp, anchor="mean", anchor_seed=3,
                                  n_sink=sink, n_recent=recent)
    idx, ko, vo = lc.run(q0, k0, v0)
    torch.cuda.synchronize()
    sc_h = lc.scores.cpu()
    ref_sc = oracle.scores(q[:, :, :S0].contiguous(), k[:, :, :S0].contiguous(), True, threads=THREADS)
    assert rel_err(sc_h, ref_sc) <= SCORE_RTOL
    ridx, _, _ = oracle.select(sc_h, budget, n_imp, 0, "mean", 3, n_sink=sink, n_recent=recent)
    assert torch.equal(idx.cpu(), ridx)
    rk, rv = oracle.compact(k[:, :, :S0].contiguous(), v[:, :, :S0].contiguous(), ridx)
    assert torch.equal(ko.cpu().view(torch.uint8), rk.view(torch.uint8))
    eager = [t.clone() for t in (idx, ko, vo)]
    lc.capture(q0, k0, v0)
    for t in (lc.idx, lc.k_out, lc.v_out):
        t.zero_()
    got = lc.replay()
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(got, eager))

    # the compressed cache goes on living: scores of the kept tokens, then one append per new token
    kept_sc = torch.gather(lc.scores, 2, idx.long()[:, None, :].expand(B, Hkv, budget))
    dc = pipeline.DecodeCache(ko, vo, kept_sc, budget, n_imp, cap, anchor="mean", anchor_seed=3, n_sink=sink,
                              n_recent=recent)
    o_k = torch.zeros(B, Hkv, cap, D, dtype=torch.bfloat16)
    o_v, o_sc = torch.zeros_like(o_k), torch.zeros(B, Hkv, cap)
    o_k[:, :, :budget], o_v[:, :, :budget], o_sc[:, :, :budget] = rk, rv, kept_sc.cpu()
    n = budget
    for step in range(steps):
        pos = S0 + step
        if n == cap:                                  # the wrapper evicts by itself; mirror it on the oracle side
            ridx, _, _ = oracle.select(dc.scores.cpu()[:, :, :n].contiguous(), budget, n_imp, 0, "mean", 3,
                                       n_sink=sink, n_recent=recent)
            new = [torch.zeros_like(t) for t in (o_k, o_v, o_sc)]
            oracle.compact_cache(o_k, o_v, o_sc, ridx, *new)
            o_k, o_v, o_sc = new
            n = budget
        dc.append(qd[:, :, pos].contiguous(), kd[:, :, pos].contiguous(), vd[:, :, pos].contiguous())
        if dc.evictions and n == budget and step and dc.n == budget + 1:
            assert torch.equal(dc._idx.cpu(), ridx), "eviction chose other tokens than the oracle on the same scores"
        o_k[:, :, n], o_v[:, :, n] = k[:, :, pos], v[:, :, pos]
        n += 1
        oracle.scores_append(q[:, :, pos].contiguous(), o_k, o_sc, n, True)
        assert dc.n == n
    torch.cuda.synchronize()
    assert dc.evictions == 2
    assert torch.equal(dc.k.cpu()[:, :, :n].view(torch.uint8), o_k[:, :, :n].view(torch.uint8))
    assert torch.equal(dc.v.cpu()[:, :, :n].view(torch.uint8), o_v[:, :, :n].view(torch.uint8))
    assert rel_err(dc.scores[:, :, :n], o_sc[:, :, :n]) <= SCORE_RTOL


# ------------------------------------------------------------------ memory layouts of Q and K
@pytest.mark.parametrize("B,Hq,Hkv,S,D,dtype,rg,W", [
    (2, 8, 2, 700, 128, "bf16", True, 0),      # ragged last tile
    (1, 4, 4, 1300, 64, "bf16", False, 0),
    (2, 4, 2, 333, 128, "f32", True, 0),
    (1, 8, 2, 2500, 128, "f16", True, 64),     # observation window, key slices
    (1, 32, 8, 4096, 128, "bf16", True, 0),    # several key blocks and chunks per row
])
def test_scores_strided_layouts(kv, oracle, B, Hq, Hkv, S, D, dtype, rg, W):
    """Q and K read in place from views: token-major projection outputs [B,S,H,D], and the first S
    tokens of longer (padded) buffers.  The oracle sees packed copies of the same values; the packed
    GPU call must agree to the bit (same arithmetic, other addresses)."""
    say(f"strided layouts B={B} Hq={Hq} Hkv={Hkv} S={S} D={D} {dtype} rg={rg} W={W}")
    w = inputs.Workload("t", B, Hq, Hkv, S, D, dtype, S // 4, 0.5, "alternating", rg, sink_bias=True)
    q, k, _ = inputs.make_qkv(w, 31)
    ref = oracle.scores(q, k, rg, threads=THREADS, window=W)
    packed, _ = kv.kvcrush_scores(q.cuda(), k.cuda(), rg, window=W)
    # token-major storage, seen as [B,H,S,D]
    q_tm = q.cuda().transpose(1, 2).contiguous().transpose(1, 2)
    k_tm = k.cuda().transpose(1, 2).contiguous().transpose(1, 2)
    assert not q_tm.is_contiguous() and q_tm.stride(2) == Hq * D
    # packed heads inside buffers of S + 77 and S + 8 tokens
    q_pad = torch.randn(B, Hq, S + 77, D, device="cuda").to(q.dtype)
    k_pad = torch.randn(B, Hkv, S + 8, D, device="cuda").to(k.dtype)
    q_pad[:, :, :S], k_pad[:, :, :S] = q.cuda(), k.cuda()
    for name, qq, kk in (("token-major", q_tm, k_tm), ("padded", q_pad[:, :, :S], k_pad[:, :, :S]),
                         ("mixed", q_tm, k_pad[:, :, :S])):
        got, _ = kv.kvcrush_scores(qq, kk, rg, window=W)
        torch.cuda.synchronize()
        assert rel_err(got, ref) <= SCORE_RTOL, name
        assert torch.equal(got, packed), name
    lse_p = kv.kvcrush_row_lse(q.cuda(), k.cuda(), window=W)
    lse_s = kv.kvcrush_row_lse(q_tm, k_pad[:, :, :S], window=W)
    torch.cuda.synchronize()
    first = max(S - W, 0) if W else 0
    assert torch.equal(lse_p[:, :, first:], lse_s[:, :, first:])


def test_scores_append_random_sweep(kv, oracle):
    """Seeded sweep of the decoding step: dtypes, head dims, group sizes, dense and paged caches,
    per-sequence device lengths, caller's softmax scale (40 cases)."""
    import random
    rng = random.Random(4242)
    for case in range(40):
        dtype = rng.choice(["bf16", "bf16", "f16", "f32"])
        td = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[dtype]
        D, Hkv, G, B = rng.choice([64, 128]), rng.choice([1, 2, 3, 8]), rng.choice([1, 2, 4, 5, 12]), rng.choice([1, 2, 3, 8])
        bs = rng.choice([16, 32])
        S = rng.choice([rng.randint(1, 70), rng.randint(1, 1200), rng.randint(1200, 3000)])
        cap = ((S + rng.randint(0, 200)) + bs - 1) // bs * bs
        rg, paged, use_len = rng.random() < 0.6, rng.random() < 0.4, rng.random() < 0.4
        scale = rng.choice([0.0, 0.0, 0.1])
        Hq = Hkv * G
        Hs = Hkv if rg else Hq
        say(f"  sweep {case}: B={B} Hq={Hq} Hkv={Hkv} S={S} cap={cap} D={D} {dtype} rg={rg} paged={paged} "
            f"block={bs} lengths={use_len} scale={scale}")
        g = torch.Generator().manual_seed(9000 + case)
        qn = torch.randn(B, Hq, D, generator=g).to(td)
        kc = torch.randn(B, Hkv, cap, D, generator=g).to(td)
        kc[:, :, :4] *= 2.0
        old = torch.rand(B, Hs, cap, generator=g) * 3.0
        lens_h = [rng.randint(1, S) for _ in range(B)] if use_len else [S] * B
        if use_len:
            lens_h[rng.randrange(B)] = S
        lens = torch.tensor(lens_h, dtype=torch.int32).cuda() if use_len else None
        kdev, kw = kc.cuda(), {}
        if paged:
            nb = cap // bs
            table = torch.randperm(B * nb, generator=g).to(torch.int32).view(B, nb)
            pool = torch.zeros(B * nb, bs, Hkv, D, dtype=td)
            pool[table.long().view(-1)] = kc.view(B, Hkv, nb, bs, D).permute(0, 2, 3, 1, 4).reshape(B * nb, bs, Hkv, D)
            kdev, kw = pool.cuda(), dict(block_table=table.cuda(), block_size=bs)
        got = kv.kvcrush_scores_append(qn.cuda(), kdev, old.clone().cuda(), S, rg, lengths=lens, scale=scale, **kw).cpu()
        for b in range(B):                     # the oracle takes one length: sequence by sequence
            n = lens_h[b]
            want = old[b:b + 1].clone().contiguous()
            oracle.scores_append(qn[b:b + 1].contiguous(), kc[b:b + 1].contiguous(), want, n, rg, scale=scale)
            assert torch.equal(got[b, :, n:], old[b, :, n:]), f"case {case}: entries beyond the length were touched"
            assert rel_err(got[b, :, :n], want[0, :, :n]) <= SCORE_RTOL, f"case {case}"


def test_thousands_of_sequences_in_one_call(kv, oracle):
    """Batch sizes in the thousands (the sequence index is a grid dimension of its own in most
    kernels): every stage and the decoding step at B = 5000, short sequences."""
    say("B = 5000 through scores, select, compact and the decoding step")
    B, Hq, Hkv, S, D, budget, n_imp = 5000, 2, 1, 40, 64, 12, 6
    w = inputs.Workload("t", B, Hq, Hkv, S, D, "bf16", budget, 0.5, "alternating", True, sink_bias=True)
    q, k, v = inputs.make_qkv(w, 77)
    sc, _ = kv.kvcrush_scores(q.cuda(), k.cuda(), True)
    idx, kind, _ = kv.kvcrush_select(sc, budget, n_imp, 0, "random", 5, n_sink=1, n_recent=2)
    ko, vo = kv.kvcrush_compact(k.cuda(), v.cuda(), idx)
    torch.cuda.synchronize()
    assert rel_err(sc, oracle.scores(q, k, True, threads=THREADS)) <= SCORE_RTOL
    ridx, rkind, _ = oracle.select(sc.cpu(), budget, n_imp, 0, "random", 5, n_sink=1, n_recent=2)
    assert torch.equal(idx.cpu(), ridx) and torch.equal(kind.cpu(), rkind)
    rk, rv = oracle.compact(k, v, ridx)
    assert torch.equal(ko.cpu().view(torch.uint8), rk.view(torch.uint8))
    assert torch.equal(vo.cpu().view(torch.uint8), rv.view(torch.uint8))
    # one decoding step on all of them
    cap = 48
    kc = torch.zeros(B, Hkv, cap, D, dtype=torch.bfloat16)
    kc[:, :, :S] = k
    old = torch.zeros(B, Hkv, cap)
    old[:, :, :S] = sc.cpu()
    qn = q[:, :, -1].contiguous()
    got = kv.kvcrush_scores_append(qn.cuda(), kc.cuda(), old.clone().cuda(), S, True)
    torch.cuda.synchronize()
    want = oracle.scores_append(qn, kc, old.clone(), S, True)
    assert rel_err(got[:, :, :S], want[:, :, :S]) <= SCORE_RTOL


def test_ragged_batch_from_padded_buffers(kv, oracle):
    """A prefill batch of unequal lengths in padded [B,H,S_max,D] buffers: one score and one select
    call per sequence on views of its own tokens (no copies of Q, K or V), one gather for the batch."""
    say("ragged batch: lengths 90, 700, 1025 in buffers padded to 1100")
    B, Hq, Hkv, D, S_max, budget, n_imp = 3, 8, 2, 128, 1100, 64, 40
    lens = [90, 700, 1025]
    w = inputs.Workload("t", B, Hq, Hkv, S_max, D, "bf16", budget, 0.5, "alternating", True, sink_bias=True)
    q, k, v = inputs.make_qkv(w, 41)
    for b, n in enumerate(lens):                       # what lies beyond a sequence's end is never read
        q[b, :, n:], k[b, :, n:], v[b, :, n:] = float("nan"), float("nan"), float("nan")
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    scores = torch.zeros(B, Hkv, S_max, device="cuda")
    idx = torch.empty(B, budget, dtype=torch.int32, device="cuda")
    for b, n in enumerate(lens):
        sc, _ = kv.kvcrush_scores(qd[b:b + 1, :, :n], kd[b:b + 1, :, :n], True)
        scores[b, :, :n] = sc[0]
        kv.kvcrush_select(scores[b:b + 1], budget, n_imp, 0, "mean", 9, want_kind=False, idx=idx[b:b + 1],
                          n_sink=2, n_recent=8, valid_len=n)
    k_out = torch.zeros(B, Hkv, budget, D, dtype=torch.bfloat16, device="cuda")
    v_out, sc_out = torch.zeros_like(k_out), torch.zeros(B, Hkv, budget, device="cuda")
    kv.kvcrush_compact_cache(kd, vd, scores, idx, k_out, v_out, sc_out)
    torch.cuda.synchronize()
    for b, n in enumerate(lens):
        qb, kb, vb = [t[b:b + 1, :, :n].contiguous() for t in (q, k, v)]
        assert rel_err(scores[b:b + 1, :, :n], oracle.scores(qb, kb, True, threads=THREADS)) <= SCORE_RTOL
        ridx, _, _ = oracle.select(scores[b:b + 1, :, :n].cpu().contiguous(), budget, n_imp, 0, "mean", 9,
                                   n_sink=2, n_recent=8)
        assert torch.equal(idx[b:b + 1].cpu(), ridx)
        rk, rv = oracle.compact(kb, vb, ridx)
        assert torch.equal(k_out[b:b + 1].cpu().view(torch.uint8), rk.view(torch.uint8))
        assert torch.equal(v_out[b:b + 1].cpu().view(torch.uint8), rv.view(torch.uint8))


def test_gathers_clamp_indices_outside_the_sequence(kv, oracle):
    """An index below 0 or at/after S is pulled to the nearest token instead of being followed
    out of the arrays (dense gather, capacity-strided gather with its scores)."""
    say("gather with out-of-range indices: clamped, not followed")
    B, Hkv, S, D = 2, 2, 300, 128
    g = torch.Generator().manual_seed(4)
    k = torch.randn(B, Hkv, S, D, generator=g).to(torch.bfloat16)
    v = torch.randn(B, Hkv, S, D, generator=g).to(torch.bfloat16)
    sc = torch.rand(B, Hkv, S, generator=g)
    idx = torch.tensor([[-7, 0, 5, 299, 300, 100000], [-2 ** 31, 1, 2, 3, 2 ** 31 - 1, 298]], dtype=torch.int32)
    good = idx.clamp(0, S - 1)
    ko, vo = kv.kvcrush_compact(k.cuda(), v.cuda(), idx.cuda(), validate=False)
    outs = [torch.zeros(B, Hkv, 8, D, dtype=torch.bfloat16, device="cuda"),
            torch.zeros(B, Hkv, 8, D, dtype=torch.bfloat16, device="cuda"), torch.zeros(B, Hkv, 8, device="cuda")]
    kv.kvcrush_compact_cache(k.cuda(), v.cuda(), sc.cuda(), idx.cuda(), *outs)
    torch.cuda.synchronize()
    rk, rv = oracle.compact(k, v, good)
    assert torch.equal(ko.cpu().view(torch.uint8), rk.view(torch.uint8))
    assert torch.equal(vo.cpu().view(torch.uint8), rv.view(torch.uint8))
    assert torch.equal(outs[0].cpu()[:, :, :6].view(torch.uint8), rk.view(torch.uint8))
    assert torch.equal(outs[2].cpu()[:, :, :6], torch.gather(sc, 2, good.long()[:, None, :].expand(B, Hkv, 6)))


@pytest.mark.parametrize("block,levels", [(64, 2), (64, 3), (128, 2), (32, 2), (1, 2)])
def test_select_on_blocks_of_alternating_sizes(kv, oracle, block, levels):
    """Score rows made of blocks of tokens that alternate between a few magnitudes: the first radix
    pass then sees whole waves leave one histogram bin for another at the same key (its ballot
    path), or lanes split over a few bins (its run-length path)."""
    say(f"select on rows of {block}-token blocks cycling through {levels} magnitudes")
    B, Hs, S = 2, 8, 16384
    g = torch.Generator().manual_seed(block * 10 + levels)
    t = torch.arange(S)
    base = (1.0 + 7.0 * ((t // block) % levels).float())[None, None, :]
    sc = (base * (1.0 + 1e-3 * torch.rand(B, Hs, S, generator=g))).contiguous()
    check_select(kv, oracle, sc, 4096, 3072, 0, "mean")
    check_select(kv, oracle, sc, 1000, 0, 6000, "alternating", n_sink=4, n_recent=60)


@pytest.mark.parametrize("B,Hs,S,budget,sink,recent", [(1, 8, 16384, 4096, 0, 0), (3, 4, 1000, 333, 4, 16), (2, 100, 700, 1, 0, 0),
                                                       (1, 8, 500, 500, 0, 0), (2, 8, 300, 48, 16, 32)])
def test_select_plain_topk_without_representatives(kv, oracle, B, Hs, S, budget, sink, recent):
    """The whole budget given to the important tokens (the baseline's own selection, Sec. 3 first
    paragraph): only the importance row is ranked.  With and without the bit words asked for."""
    say(f"plain top-n B={B} Hs={Hs} S={S} budget={budget} sink={sink} recent={recent}")
    sc = inputs.make_scores(B, Hs, S, seed=S + budget, ties=True)
    n_imp = budget - sink - recent
    ridx, rkind, rbits = oracle.select(sc, budget, n_imp, 0, "mean", 1, n_sink=sink, n_recent=recent)
    idx, kind, _ = kv.kvcrush_select(sc.cuda(), budget, n_imp, 0, "mean", 1, n_sink=sink, n_recent=recent)
    idx2, kind2, bits2 = kv.kvcrush_select(sc.cuda(), budget, n_imp, 0, "mean", 1, n_sink=sink, n_recent=recent,
                                           want_bits=True)
    torch.cuda.synchronize()
    assert torch.equal(idx.cpu(), ridx) and torch.equal(kind.cpu(), rkind)
    assert torch.equal(idx2.cpu(), ridx) and torch.equal(kind2.cpu(), rkind) and torch.equal(bits2.cpu(), rbits)
