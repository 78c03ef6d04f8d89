"""Pins for the oracle's score stage (Alg. 1's attention weights, read as the
attention each token receives).  None of these re-type the oracle's loop: they
are a brute force that materialises the full S x S matrix in pure Python,
closed forms, invariants, and a float64 library softmax."""
import math
from fractions import Fraction

import pytest
import torch

from paper_2503_00022_amd import inputs


def brute_force_colsums(q, k, G):
    """Pure-Python: build every head's full attention matrix, then add columns."""
    B, Hq, S, D = q.shape
    out = [[[0.0] * S for _ in range(Hq)] for _ in range(B)]
    ql, kl = q.double().tolist(), k.double().tolist()
    for b in range(B):
        for h in range(Hq):
            A = [[0.0] * S for _ in range(S)]
            for i in range(S):
                logits = []
                for j in range(i + 1):
                    logits.append(sum(ql[b][h][i][d] * kl[b][h // G][j][d] for d in range(D)) / math.sqrt(D))
                mx = max(logits)
                e = [math.exp(x - mx) for x in logits]
                tot = math.fsum(e)
                for j in range(i + 1):
                    A[i][j] = e[j] / tot
            for t in range(S):
                out[b][h][t] = math.fsum(A[i][t] for i in range(S))
    return torch.tensor(out, dtype=torch.float64)


@pytest.mark.parametrize("S,Hq,Hkv,D,dtype", [(16, 4, 4, 8, torch.float32), (13, 4, 2, 16, torch.bfloat16),
                                              (7, 2, 1, 4, torch.float32), (1, 1, 1, 8, torch.float32)])
def test_brute_force_full_matrix(oracle, S, Hq, Hkv, D, dtype):
    g = torch.Generator().manual_seed(S * 100 + Hq)
    q = torch.randn(2, Hq, S, D, generator=g).to(dtype)
    k = torch.randn(2, Hkv, S, D, generator=g).to(dtype)
    G = Hq // Hkv
    ref = brute_force_colsums(q, k, G)
    got = oracle.scores(q, k, reduce_groups=False).double()
    assert torch.allclose(got, ref, rtol=2e-7, atol=0)
    # group reduction = plain sum of the group's heads
    got_g = oracle.scores(q, k, reduce_groups=True).double()
    ref_g = ref.view(2, Hkv, G, S).sum(dim=2)
    assert torch.allclose(got_g, ref_g, rtol=2e-7, atol=0)


def test_uniform_attention_closed_form(oracle):
    """Q = 0 makes every causal row uniform, so token t (0-based) receives
    sum_{i=t+1}^{S} 1/i = H_S - H_t.  S = 4 gives 25/12, 13/12, 7/12, 1/4."""
    S, D = 4, 8
    q = torch.zeros(1, 1, S, D)
    k = torch.randn(1, 1, S, D, generator=torch.Generator().manual_seed(1))
    got = oracle.scores(q, k, reduce_groups=False)[0, 0].double()
    want = torch.tensor([25 / 12, 13 / 12, 7 / 12, 1 / 4], dtype=torch.float64)
    assert torch.allclose(got, want, rtol=1e-7)
    # and a longer one against exact rationals
    S = 97
    q = torch.zeros(1, 1, S, D)
    k = torch.randn(1, 1, S, D, generator=torch.Generator().manual_seed(2))
    got = oracle.scores(q, k, reduce_groups=False)[0, 0].double()
    want = torch.tensor([float(sum(Fraction(1, i) for i in range(t + 1, S + 1))) for t in range(S)],
                        dtype=torch.float64)
    assert torch.allclose(got, want, rtol=1e-6)


def test_equal_keys_also_uniform(oracle):
    S, D = 33, 16
    g = torch.Generator().manual_seed(3)
    q = torch.randn(1, 2, S, D, generator=g)
    k = torch.randn(1, 1, 1, D, generator=g).expand(1, 2, S, D).contiguous()
    got = oracle.scores(q, k, reduce_groups=False).double()
    want = torch.tensor([sum(1.0 / i for i in range(t + 1, S + 1)) for t in range(S)], dtype=torch.float64)
    assert torch.allclose(got[0, 0], want, rtol=1e-6) and torch.allclose(got[0, 1], want, rtol=1e-6)


def test_single_token(oracle):
    q = torch.randn(1, 3, 1, 8, generator=torch.Generator().manual_seed(4))
    k = torch.randn(1, 3, 1, 8, generator=torch.Generator().manual_seed(5))
    assert torch.equal(oracle.scores(q, k, reduce_groups=False), torch.ones(1, 3, 1))


def test_dominant_key_takes_all_later_rows(oracle):
    """If one key's logit dwarfs the others for every query, rows j* .. S-1 put
    all their mass on it: c[j*] ~= S - j*."""
    S, D, js = 40, 8, 11
    q = torch.zeros(1, 1, S, D)
    q[..., 0] = 1.0
    k = torch.zeros(1, 1, S, D)
    k[0, 0, js, 0] = 200.0            # logit 200/sqrt(8) ~ 70 above the rest
    got = oracle.scores(q, k, reduce_groups=False)[0, 0].double()
    assert abs(got[js].item() - (S - js)) < 1e-9 * S
    # earlier tokens only get the uniform rows before js
    want0 = sum(1.0 / i for i in range(1, js + 1))
    assert abs(got[0].item() - want0) < 1e-6


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_column_sums_total_the_number_of_rows(oracle, dtype):
    w = inputs.Workload("t", 2, 8, 2, 200, 32, "bf16" if dtype == torch.bfloat16 else "f32", 50, 0.5,
                        "alternating", False, sink_bias=True)
    q, k, _ = inputs.make_qkv(w, 7)
    sc = oracle.scores(q, k, reduce_groups=False).double()
    assert torch.allclose(sc.sum(-1), torch.full((2, 8), 200.0, dtype=torch.float64), rtol=1e-6)
    scg = oracle.scores(q, k, reduce_groups=True).double()
    assert torch.allclose(scg.sum(-1), torch.full((2, 2), 4 * 200.0, dtype=torch.float64), rtol=1e-6)
    assert (sc > 0).all()


def library_colsums(q, k, G):
    """float64 library softmax over the masked logits, summed over query rows."""
    qd, kd = q.double(), k.double().repeat_interleave(G, dim=1)
    S, D = q.shape[-2:]
    logits = qd @ kd.transpose(-1, -2) / math.sqrt(D)
    mask = torch.ones(S, S, dtype=torch.bool).tril()
    logits = logits.masked_fill(~mask, float("-inf"))
    A = torch.softmax(logits, dim=-1)
    return A.sum(dim=-2), torch.logsumexp(logits, dim=-1), A


@pytest.mark.parametrize("S,Hq,Hkv,D,dtype", [(384, 8, 2, 64, torch.bfloat16), (512, 4, 4, 64, torch.float32),
                                              (257, 4, 1, 128, torch.bfloat16), (300, 4, 2, 128, torch.float16)])
def test_against_library_softmax(oracle, S, Hq, Hkv, D, dtype):
    w = inputs.Workload("t", 1, Hq, Hkv, S, D, {torch.bfloat16: "bf16", torch.float16: "f16", torch.float32: "f32"}[dtype],
                        64, 0.5, "alternating", False, sink_bias=True)
    q, k, _ = inputs.make_qkv(w, 11)
    G = Hq // Hkv
    ref, ref_lse, A = library_colsums(q, k, G)
    got, lse = oracle.scores(q, k, reduce_groups=False, want_lse=True)
    assert torch.allclose(got.double(), ref, rtol=3e-7, atol=0)
    assert torch.allclose(lse.double(), ref_lse, rtol=0, atol=2e-6)
    # the last token is seen by the last query only: its score is one probability
    assert torch.allclose(got[..., -1].double(), A[..., -1, -1], rtol=2e-7)
    # threaded path == single-threaded path, bit for bit
    got_t, lse_t = oracle.scores(q, k, reduce_groups=False, want_lse=True, threads=4)
    assert torch.equal(got_t, got) and torch.equal(lse_t, lse)
    gr = oracle.scores(q, k, reduce_groups=True)
    gr_t = oracle.scores(q, k, reduce_groups=True, threads=3)
    assert torch.equal(gr, gr_t)
    assert torch.allclose(gr.double(), ref.view(1, Hkv, G, S).sum(2), rtol=3e-7)


def test_row_ranges_add_up(oracle):
    g = torch.Generator().manual_seed(12)
    q = torch.randn(64, 16, generator=g).to(torch.bfloat16)
    k = torch.randn(64, 16, generator=g).to(torch.bfloat16)
    full = oracle.head_colsums(q, k)
    parts = oracle.head_colsums(q, k, 0, 20) + oracle.head_colsums(q, k, 20, 64)
    assert torch.allclose(full, parts, rtol=1e-14)
    # rows before t never reach token t
    late = oracle.head_colsums(q, k, 0, 30)
    assert (late[30:] == 0).all()


# ------------------------------------------------------------ observation window
def test_window_matches_brute_force_and_library(oracle):
    """Only the last W query rows contribute: rows of the full attention matrix
    are summed from S-W on (brute force), and a float64 library softmax agrees."""
    g = torch.Generator().manual_seed(21)
    S, W = 14, 5
    q = torch.randn(1, 2, S, 8, generator=g)
    k = torch.randn(1, 1, S, 8, generator=g)
    _, _, A = library_colsums(q, k, 2)
    want = A[..., S - W:, :].sum(dim=-2)
    got = oracle.scores(q, k, reduce_groups=False, window=W).double()
    assert torch.allclose(got, want, rtol=3e-7)
    # every head's scores now total W; W >= S and W = 0 mean "all rows"
    assert torch.allclose(got.sum(-1), torch.full((1, 2), float(W), dtype=torch.float64), rtol=1e-6)
    full = oracle.scores(q, k, reduce_groups=False)
    assert torch.equal(oracle.scores(q, k, reduce_groups=False, window=S), full)
    assert torch.equal(oracle.scores(q, k, reduce_groups=False, window=S + 7), full)
    # W = 1: the last row of the attention matrix itself
    one = oracle.scores(q, k, reduce_groups=False, window=1).double()
    assert torch.allclose(one, A[..., -1, :], rtol=3e-7)
    # group reduction and the threaded path agree with it
    gr = oracle.scores(q, k, reduce_groups=True, window=W).double()
    assert torch.allclose(gr[:, 0], want.sum(1), rtol=3e-7)
    assert torch.equal(oracle.scores(q, k, reduce_groups=True, window=W, threads=2).double(), gr)
    # lse is reported for the window rows only
    _, lse = oracle.scores(q, k, reduce_groups=False, want_lse=True, window=W)
    assert (lse[..., : S - W] == 0).all() and (lse[..., S - W:] != 0).all()


def test_maxpool_matches_library(oracle):
    g = torch.Generator().manual_seed(22)
    x = torch.randn(3, 4, 37, generator=g)
    for kernel in (1, 3, 5, 7, 41):
        want = torch.nn.functional.max_pool1d(x.view(12, 1, 37), kernel, stride=1, padding=kernel // 2).view(3, 4, 37)
        assert torch.equal(oracle.maxpool(x, kernel), want)
    # hand-worked: kernel 3 on 1 5 2 0 4 -> 5 5 5 4 4
    assert oracle.maxpool(torch.tensor([[1.0, 5.0, 2.0, 0.0, 4.0]]), 3).tolist() == [[5.0, 5.0, 5.0, 4.0, 4.0]]


def test_explicit_scale_and_zero_padding(oracle):
    """A caller-supplied scale replaces 1/sqrt(D): heads of 24 values zero-padded to 32 and scored with
    1/sqrt(24) give what the unpadded heads give, and the default is 1/sqrt(D)."""
    g = torch.Generator().manual_seed(31)
    S, D, Dp = 50, 24, 32
    q = torch.randn(1, 2, S, D, generator=g)
    k = torch.randn(1, 1, S, D, generator=g)
    pad = lambda t: torch.cat([t, torch.zeros(*t.shape[:-1], Dp - D)], dim=-1).contiguous()
    plain = oracle.scores(q, k, False)
    assert torch.equal(oracle.scores(q, k, False, scale=1.0 / math.sqrt(D)), plain)
    assert torch.allclose(oracle.scores(pad(q), pad(k), False, scale=1.0 / math.sqrt(D)).double(), plain.double(),
                          rtol=1e-6)
    assert not torch.allclose(oracle.scores(pad(q), pad(k), False), plain, rtol=1e-3)   # 1/sqrt(32) is another method
    # a library softmax with the same scale
    logits = (q.double() @ k.double().repeat_interleave(2, 1).transpose(-1, -2)) * 0.3
    logits = logits.masked_fill(~torch.ones(S, S, dtype=torch.bool).tril(), float("-inf"))
    assert torch.allclose(oracle.scores(q, k, False, scale=0.3).double(), torch.softmax(logits, -1).sum(-2), rtol=3e-7)


def test_half_precision_inputs_are_widened_exactly(oracle):
    """fp16 inputs, subnormals included (values near 1e-6 have no normal fp16 form): with Q = the unit
    vector e_0 times 1024 and K[:, 0] = the value under test, the last attention row is the softmax of
    1024 / sqrt(D) times those values, which the library computes from the same halves widened by torch."""
    S, D = 64, 16
    vals = torch.cat([torch.tensor([0.0, -0.0, 6.0e-8, -6.0e-8, 5.9e-5, 6.2e-5, 1.0, -2.5, 65504.0 / 4096]),
                      torch.randn(S - 9, generator=torch.Generator().manual_seed(6)) * 1e-5]).to(torch.float16)
    q = torch.zeros(1, 1, S, D, dtype=torch.float16)
    q[..., 0] = 1024.0
    k = torch.zeros(1, 1, S, D, dtype=torch.float16)
    k[0, 0, :, 0] = vals
    got = oracle.scores(q, k, False, window=1).double()[0, 0]
    want = torch.softmax(vals.double() * 1024.0 / math.sqrt(D), dim=0)
    assert torch.allclose(got, want, rtol=3e-7)
