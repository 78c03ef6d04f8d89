"""Pins for the oracle's decoding-time steps: appending one query row to the
running received-attention scores, and the eviction gather on capacity-strided
caches.  The chief pin is an identity: a prefix scored at once plus one append
per later token equals the whole sequence scored at once (column sums of the
causal attention matrix, split by rows)."""
import math

import pytest
import torch


def fresh_cache(B, H, cap, D, dtype, fill):
    return torch.full((B, H, cap, D), fill, dtype=dtype)


@pytest.mark.parametrize("Hq,Hkv,D,dtype,rg", [(4, 2, 16, torch.float32, True), (4, 2, 16, torch.bfloat16, False),
                                               (3, 3, 8, torch.float32, False), (6, 1, 32, torch.bfloat16, True)])
def test_prefix_plus_appends_equals_whole_sequence(oracle, Hq, Hkv, D, dtype, rg):
    B, S0, S, cap = 2, 9, 23, 40
    g = torch.Generator().manual_seed(Hq * 10 + D)
    q = torch.randn(B, Hq, S, D, generator=g).to(dtype)
    k = torch.randn(B, Hkv, S, D, generator=g).to(dtype)
    Hs = Hkv if rg else Hq
    whole = oracle.scores(q, k, rg)
    kc = fresh_cache(B, Hkv, cap, D, dtype, 7.0)            # junk beyond the valid length must not matter
    kc[:, :, :S] = k
    sc = torch.full((B, Hs, cap), -123.0)                   # sentinel: entries at or beyond S stay untouched
    sc[:, :, :S0] = oracle.scores(q[:, :, :S0].contiguous(), k[:, :, :S0].contiguous(), rg)
    for n in range(S0 + 1, S + 1):
        oracle.scores_append(q[:, :, n - 1].contiguous(), kc, sc, n, rg)
        assert (sc[:, :, n:] == -123.0).all()
        # each step adds one probability row per head: the total grows by the number of heads summed
        per_row = (Hq // Hkv if rg else 1)
        assert torch.allclose(sc[:, :, :n].double().sum(-1), torch.full((B, Hs), float(per_row * n), dtype=torch.float64),
                              rtol=1e-5)
    assert torch.allclose(sc[:, :, :S], whole, rtol=2e-5, atol=0)


def test_append_is_one_library_softmax_row(oracle):
    B, Hq, Hkv, D, S, cap = 1, 4, 2, 32, 50, 64
    g = torch.Generator().manual_seed(5)
    qn = torch.randn(B, Hq, D, generator=g)
    kc = torch.randn(B, Hkv, cap, D, generator=g)
    old = torch.rand(B, Hq, cap, generator=g)
    sc = old.clone()
    oracle.scores_append(qn, kc, sc, S, False)
    logits = torch.einsum("bhd,bhsd->bhs", qn.double(), kc[:, :, :S].double().repeat_interleave(2, dim=1)) / math.sqrt(D)
    p = torch.softmax(logits, dim=-1)
    want = old.clone().double()
    want[:, :, :S - 1] += p[:, :, :S - 1]
    want[:, :, S - 1] = p[:, :, S - 1]                      # the new token's slot is overwritten, not added to
    assert torch.allclose(sc.double(), want, rtol=2e-7)
    assert torch.equal(sc[:, :, S:], old[:, :, S:])
    # grouped: the two heads of a KV group add up
    scg = old[:, :Hkv].clone()
    oracle.scores_append(qn, kc, scg, S, True)
    wantg = old[:, :Hkv].clone().double()
    pg = p.view(B, Hkv, 2, S).sum(2)
    wantg[:, :, :S - 1] += pg[:, :, :S - 1]
    wantg[:, :, S - 1] = pg[:, :, S - 1]
    assert torch.allclose(scg.double(), wantg, rtol=2e-7)


def test_append_with_a_caller_scale_is_the_library_softmax_at_that_scale(oracle):
    """`scale` replaces 1/sqrt(D) as the factor on q . k (models with an attention scale of their own;
    zero-padded heads scored with 1/sqrt(true size)).  Pinned by a float64 library softmax at that
    scale, by scale = 1/sqrt(D) being the default spelled out, and by padding: a head zero-padded
    from 24 to 32 values with scale 1/sqrt(24) scores as the 24-value head does by default."""
    B, Hq, Hkv, D, S, cap = 2, 4, 2, 24, 37, 40
    g = torch.Generator().manual_seed(8)
    qn = torch.randn(B, Hq, D, generator=g)
    kc = torch.randn(B, Hkv, cap, D, generator=g)
    old = torch.rand(B, Hq, cap, generator=g)
    dots = torch.einsum("bhd,bhsd->bhs", qn.double(), kc[:, :, :S].double().repeat_interleave(2, dim=1))
    for scale in (0.37, 1.0, 1.0 / math.sqrt(D)):
        sc = old.clone()
        oracle.scores_append(qn, kc, sc, S, False, scale=scale)
        p = torch.softmax(dots * scale, dim=-1)
        want = old.clone().double()
        want[:, :, :S - 1] += p[:, :, :S - 1]
        want[:, :, S - 1] = p[:, :, S - 1]
        assert torch.allclose(sc.double(), want, rtol=2e-7), f"scale {scale}"
        assert torch.equal(sc[:, :, S:], old[:, :, S:])
    default = oracle.scores_append(qn, kc, old.clone(), S, False)
    spelled = oracle.scores_append(qn, kc, old.clone(), S, False, scale=1.0 / math.sqrt(D))
    assert torch.equal(default, spelled)
    # a different scale really gives different probabilities (the argument is not ignored)
    other = oracle.scores_append(qn, kc, old.clone(), S, False, scale=0.37)
    assert not torch.allclose(other, default, rtol=1e-3)
    qp = torch.zeros(B, Hq, 32); qp[..., :D] = qn
    kp = torch.zeros(B, Hkv, cap, 32); kp[..., :D] = kc
    padded = oracle.scores_append(qp, kp, old.clone(), S, False, scale=1.0 / math.sqrt(D))
    assert torch.allclose(padded, default, rtol=1e-6)


def test_append_first_token(oracle):
    """S = 1: the only key gets probability one from every head."""
    qn = torch.randn(1, 4, 8, generator=torch.Generator().manual_seed(1))
    kc = torch.randn(1, 2, 5, 8, generator=torch.Generator().manual_seed(2))
    sc = torch.full((1, 2, 5), 9.0)
    oracle.scores_append(qn, kc, sc, 1, True)
    assert sc[0, :, 0].tolist() == [2.0, 2.0] and (sc[0, :, 1:] == 9.0).all()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_compact_cache_is_a_strided_gather(oracle, dtype):
    B, Hkv, Hs, D, cap_src, cap_dst, budget = 2, 3, 5, 16, 30, 20, 11
    g = torch.Generator().manual_seed(3)
    k = torch.randn(B, Hkv, cap_src, D, generator=g).to(dtype)
    v = torch.randn(B, Hkv, cap_src, D, generator=g).to(dtype)
    sc = torch.randn(B, Hs, cap_src, generator=g)
    idx = torch.stack([torch.randperm(cap_src, generator=g)[:budget].sort().values for _ in range(B)]).to(torch.int32)
    ko, vo = torch.full((B, Hkv, cap_dst, D), 5.0, dtype=dtype), torch.full((B, Hkv, cap_dst, D), 6.0, dtype=dtype)
    so = torch.full((B, Hs, cap_dst), 7.0)
    oracle.compact_cache(k, v, sc, idx, ko, vo, so)
    li = idx.long()
    assert torch.equal(ko[:, :, :budget], torch.gather(k, 2, li[:, None, :, None].expand(B, Hkv, budget, D)))
    assert torch.equal(vo[:, :, :budget], torch.gather(v, 2, li[:, None, :, None].expand(B, Hkv, budget, D)))
    assert torch.equal(so[:, :, :budget], torch.gather(sc, 2, li[:, None, :].expand(B, Hs, budget)))
    assert (ko[:, :, budget:] == 5.0).all() and (vo[:, :, budget:] == 6.0).all() and (so[:, :, budget:] == 7.0).all()
    # same result as the dense gather of stage 5 when the strides are the lengths
    rk, rv = oracle.compact(k, v, idx)
    assert torch.equal(rk, ko[:, :, :budget]) and torch.equal(rv, vo[:, :, :budget])
