"""Pins for the oracle's selection stages: top-k, head-behaviour bits (Alg. 1),
anchors, Hamming grouping and representatives (Alg. 2), and the final index
list.  The checks are an independent pure-Python brute force (pairwise Hamming
medoid, sorted() with an explicit key), hand-worked examples from
tests/golden/hamming_examples.txt, splitmix64's published outputs, and
structural invariants."""
import os
import random

import numpy as np
import pytest
import torch

from paper_2503_00022_amd import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hamming_examples.txt")


# ---------------------------------------------------------------- helpers
def py_topk(vals, k):
    return sorted(range(len(vals)), key=lambda i: (-vals[i], i))[:k]


def popcount(x):
    return bin(x).count("1")


def py_group(bits, important, Br, anchor):
    """Alg. 2, brute force: medoid by pairwise Hamming distances."""
    disc = [t for t in range(len(bits)) if t not in important]
    N = len(disc)
    order = sorted(disc, key=lambda t: (popcount(bits[t] ^ anchor), t))
    reps = []
    for j in range(Br):
        members = order[j * N // Br:(j + 1) * N // Br]
        cost = {t: sum(popcount(bits[t] ^ bits[u]) for u in members) for t in members}
        reps.append(min(members, key=lambda t: (cost[t], t)))
    return reps, order


def py_select(sc, budget, n_imp, kbit, anchor_fn):
    Hs, S = len(sc), len(sc[0])
    bits = [0] * S
    for r in range(Hs):
        for t in py_topk(sc[r], kbit):
            bits[t] |= 1 << r
    imp = []
    for t in range(S):
        acc = np.float32(0.0)
        for r in range(Hs):
            acc = np.float32(acc + np.float32(sc[r][t]))
        imp.append(float(acc))
    important = set(py_topk(imp, n_imp))
    anchor = anchor_fn(bits, important)
    reps, _ = py_group(bits, important, budget - n_imp, anchor)
    idx = sorted(important | set(reps))
    kind = [1 if t in reps else 0 for t in idx]
    return idx, kind, bits


def words_to_int(row):
    v = 0
    for w, x in enumerate(row.tolist()):
        v |= (x & (2**64 - 1)) << (64 * w)
    return v


def int_to_words(v, W):
    out = []
    for w in range(W):
        x = (v >> (64 * w)) & (2**64 - 1)
        out.append(x - 2**64 if x >= 2**63 else x)
    return out


def alternating(Hs):
    return sum(1 << r for r in range(Hs) if r & 1)


# ---------------------------------------------------------------- top-k
def test_topk_matches_full_sort_with_ties(oracle):
    rng = random.Random(0)
    for n in [1, 2, 17, 100, 1000]:
        for _ in range(5):
            vals = [float(rng.randint(0, 6)) * 0.25 for _ in range(n)]  # many duplicates
            v = torch.tensor(vals)
            for k in {0, 1, n // 3, n - 1 if n > 1 else 1, n}:
                assert oracle.topk(v, k).tolist() == py_topk(vals, k)


def test_topk_tie_straddling_threshold(oracle):
    v = torch.tensor([1.0, 5.0, 3.0, 3.0, 3.0, 0.5, 3.0])
    assert oracle.topk(v, 3).tolist() == [1, 2, 3]      # two of the four 3.0s: lowest indices
    assert oracle.topk(v, 1).tolist() == [1]
    assert sorted(oracle.topk(v, 7).tolist()) == list(range(7))


# ---------------------------------------------------------------- bits
@pytest.mark.parametrize("Hs,S,kbit", [(4, 50, 10), (33, 80, 41), (64, 64, 1), (70, 30, 30), (128, 40, 7)])
def test_bits_membership_roundtrip(oracle, Hs, S, kbit):
    sc = inputs.make_scores(1, Hs, S, seed=Hs * S, ties=True)[0]
    bw = oracle.bits(sc, kbit)
    assert bw.shape == (S, (Hs + 63) // 64)
    ints = [words_to_int(bw[t]) for t in range(S)]
    for r in range(Hs):
        members = [t for t in range(S) if (ints[t] >> r) & 1]
        assert len(members) == kbit                                  # exactly kbit ones per head
        assert members == sorted(py_topk(sc[r].tolist(), kbit))
    assert sum(popcount(x) for x in ints) == Hs * kbit
    assert all(x < (1 << Hs) for x in ints)                          # no stray bits above Hs


# ---------------------------------------------------------------- anchors
def test_splitmix64_published_outputs(oracle):
    # first outputs of splitmix64 seeded with 0, as published with the generator
    assert oracle.splitmix64(0, 3) == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]


def test_anchor_modes(oracle):
    S = 12
    for Hs in [4, 8, 32, 33, 64, 100]:
        W = (Hs + 63) // 64
        bw = torch.zeros(S, W, dtype=torch.int64)
        imp = torch.zeros(S, dtype=torch.uint8)
        _, a = oracle.group(Hs, bw, imp, 2, anchor="alternating")
        assert words_to_int(a) == alternating(Hs)
        assert words_to_int(a) == (0xAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAA & ((1 << Hs) - 1))
        for seed, b in [(0, 0), (123456789, 3)]:
            _, a = oracle.group(Hs, bw, imp, 2, anchor="random", anchor_seed=seed, batch_index=b)
            z = oracle.splitmix64(seed + b, W)
            want = sum(z[w] << (64 * w) for w in range(W)) & ((1 << Hs) - 1)
            assert words_to_int(a) == want
    # random anchor for seed 0, batch 0, 8 heads: low byte of the published first output
    _, a = oracle.group(8, torch.zeros(S, 1, dtype=torch.int64), torch.zeros(S, dtype=torch.uint8), 1,
                        anchor="random", anchor_seed=0)
    assert words_to_int(a) == 0xAF


def test_mean_anchor_strict_majority_over_discarded_only(oracle):
    # H = 3.  discarded tokens 1..5; token 0 is important and must not vote.
    # bit0 set in 3 of 5 -> 1 ; bit1 set in 2 of 5 -> 0 ; bit2: 0
    bits = [0b111, 0b001, 0b001, 0b011, 0b010, 0b000]
    bw = torch.tensor([[b] for b in bits], dtype=torch.int64)
    imp = torch.tensor([1, 0, 0, 0, 0, 0], dtype=torch.uint8)
    _, a = oracle.group(3, bw, imp, 1, anchor="mean")
    assert words_to_int(a) == 0b001
    # exactly half is not a majority: 4 discarded, bit0 set in 2 -> 0
    bits = [0b1, 0b1, 0b1, 0b0, 0b0]
    bw = torch.tensor([[b] for b in bits], dtype=torch.int64)
    imp = torch.tensor([1, 0, 0, 0, 0], dtype=torch.uint8)
    _, a = oracle.group(1, bw, imp, 1, anchor="mean")
    assert words_to_int(a) == 0


# ---------------------------------------------------------------- Alg. 2
def parse_golden():
    kv = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                key, val = line.split("=", 1)
                kv[key.strip()] = val.strip()
    return kv


def test_hand_worked_examples(oracle):
    g = parse_golden()
    H, S = int(g["H"]), int(g["S"])
    bits = [0] * S
    for item in g["bits"].split():
        t, s = item.split(":")
        bits[int(t)] = int(s, 2)
    important = [int(x) for x in g["important"].split()]
    assert int(g["anchor"], 2) == alternating(H)
    bw = torch.tensor([[b] for b in bits], dtype=torch.int64)
    imp = torch.zeros(S, dtype=torch.uint8)
    imp[important] = 1
    # the fixture's own intermediate values hold for the brute force
    _, order = py_group(bits, set(important), 2, int(g["anchor"], 2))
    assert order == [int(x) for x in g["order"].split()]
    for item in g["distance"].split():
        t, d = item.split(":")
        assert popcount(bits[int(t)] ^ int(g["anchor"], 2)) == int(d)
    for ex in ("ex1", "ex2", "ex3"):
        Br = int(g[f"{ex}_Br"])
        reps, a = oracle.group(H, bw, imp, Br, anchor="alternating")
        assert reps.tolist() == [int(x) for x in g[f"{ex}_reps"].split()]
        assert sorted(important + reps.tolist()) == [int(x) for x in g[f"{ex}_idx"].split()]


@pytest.mark.parametrize("Hs", [3, 8, 32, 40, 65, 128])
def test_group_matches_pairwise_hamming_brute_force(oracle, Hs):
    rng = random.Random(Hs)
    W = (Hs + 63) // 64
    for trial in range(6):
        S = rng.randint(5, 70)
        density = rng.choice([0.15, 0.5, 0.85])
        bits = [sum(1 << r for r in range(Hs) if rng.random() < density) for _ in range(S)]
        if trial == 0:
            bits = [bits[0]] * S                                     # all vectors equal
        n_imp = rng.randint(0, S - 1)
        important = set(rng.sample(range(S), n_imp))
        N = S - n_imp
        Br = rng.randint(1, N)
        bw = torch.tensor([int_to_words(b, W) for b in bits], dtype=torch.int64)
        imp = torch.zeros(S, dtype=torch.uint8)
        imp[list(important)] = 1
        for mode in ("alternating", "random", "mean", "explicit"):
            kw = {}
            if mode == "alternating":
                anchor = alternating(Hs)
            elif mode == "random":
                z = oracle.splitmix64(99 + trial, W)
                anchor = sum(z[w] << (64 * w) for w in range(W)) & ((1 << Hs) - 1)
                kw = dict(anchor_seed=99, batch_index=trial)
            elif mode == "mean":
                disc = [t for t in range(S) if t not in important]
                anchor = sum(1 << r for r in range(Hs) if 2 * sum((bits[t] >> r) & 1 for t in disc) > N)
            else:
                anchor = rng.getrandbits(Hs)
                kw = dict(anchor_explicit=torch.tensor(int_to_words(anchor, W), dtype=torch.int64))
            want, order = py_group(bits, important, Br, anchor)
            reps, a = oracle.group(Hs, bw, imp, Br, anchor=mode, **kw)
            assert words_to_int(a) == anchor
            assert reps.tolist() == want
            if trial == 0:   # equal vectors: first (lowest) token of each rank range
                assert want == [min(order[j * N // Br:(j + 1) * N // Br]) for j in range(Br)]


def test_bucket_sizes_differ_by_at_most_one():
    for N in [1, 7, 100, 13312, 32000]:
        for Br in [1, 3, 64, 1024]:
            if Br > N:
                continue
            sizes = [(j + 1) * N // Br - j * N // Br for j in range(Br)]
            assert sum(sizes) == N and max(sizes) - min(sizes) <= 1 and min(sizes) >= 1


# ---------------------------------------------------------------- whole selection
@pytest.mark.parametrize("B,Hs,S,budget,n_imp,kbit,anchor,ties", [
    (2, 8, 120, 30, 15, 0, "alternating", True),
    (1, 32, 200, 64, 48, 0, "random", False),
    (2, 4, 90, 40, 10, 60, "mean", True),       # kbit > S/2: the mean anchor has one-bits
    (1, 70, 64, 20, 0, 0, "alternating", True), # no important tokens: everything is grouped
    (1, 8, 64, 20, 20, 0, "mean", False),       # no representatives: plain top-k
    (1, 5, 33, 33, 11, 0, "random", True),      # budget == S: identity
])
def test_select_matches_brute_force(oracle, B, Hs, S, budget, n_imp, kbit, anchor, ties):
    sc = inputs.make_scores(B, Hs, S, seed=S + Hs, ties=ties)
    idx, kind, bw = oracle.select(sc, budget, n_imp, kbit, anchor, anchor_seed=5)
    kb = kbit or budget
    W = (Hs + 63) // 64
    for b in range(B):
        def anchor_fn(bits, important):
            if anchor == "alternating":
                return alternating(Hs)
            if anchor == "random":
                z = oracle.splitmix64(5 + b, W)
                return sum(z[w] << (64 * w) for w in range(W)) & ((1 << Hs) - 1)
            disc = [t for t in range(S) if t not in important]
            return sum(1 << r for r in range(Hs) if 2 * sum((bits[t] >> r) & 1 for t in disc) > len(disc))
        want_idx, want_kind, want_bits = py_select(sc[b].tolist(), budget, n_imp, kb, anchor_fn)
        assert idx[b].tolist() == want_idx
        assert kind[b].tolist() == want_kind
        assert [words_to_int(bw[b, t]) for t in range(S)] == want_bits
        # invariants of the final cache
        assert len(set(idx[b].tolist())) == budget
        assert all(x < y for x, y in zip(idx[b].tolist(), idx[b].tolist()[1:]))
        assert int((kind[b] == 0).sum()) == n_imp and int((kind[b] == 1).sum()) == budget - n_imp
    if anchor == "mean" and kbit > S // 2:
        # make sure the one-branch of the majority vote was really exercised
        assert anchor_fn(want_bits, set(t for t, kd in zip(want_idx, want_kind) if kd == 0)) != 0
    if budget == S:
        assert idx[0].tolist() == list(range(S))
    if n_imp == budget:
        imp = sc[0].clone()
        acc = torch.zeros(S)
        for r in range(Hs):
            acc = acc + imp[r]
        assert sorted(py_topk(acc.tolist(), budget)) == idx[0].tolist()


def test_importance_sum_is_sequential_fp32(oracle):
    """Row order of the fp32 sum decides a top-1: (1e8 + -1e8) + 1 = 1 but
    1e8 + (-1e8 + 1) = 0 in fp32."""
    S = 4
    sc = torch.zeros(1, 3, S)
    sc[0, :, 0] = torch.tensor([1e8, -1e8, 1.0])     # sequential sum = 1.0
    sc[0, :, 1] = torch.tensor([0.25, 0.25, 0.25])   # 0.75
    sc[0, :, 2] = torch.tensor([2.0, 1e8, -1e8])     # (2+1e8) - 1e8 = 0 in fp32, but 2 in wider arithmetic
    idx, kind, _ = oracle.select(sc, 1, 1, 1, "alternating")
    assert idx.tolist() == [[0]]


def test_mean_anchor_is_zero_under_2x_compression(oracle):
    """With exact per-head top-k and kbit <= S/2 no head has a majority of ones
    among the discarded tokens, so the mean anchor is the zero vector and the
    distance is the popcount itself."""
    sc = inputs.make_scores(1, 8, 256, seed=1)
    idx, kind, bw = oracle.select(sc, 64, 48, 0, "mean")
    imp = torch.zeros(256, dtype=torch.uint8)
    imp[idx[0][kind[0] == 0].long()] = 1
    _, a = oracle.group(8, bw[0], imp, 16, anchor="mean")
    assert words_to_int(a) == 0


# ---------------------------------------------------------------- protected ends
@pytest.mark.parametrize("B,Hs,S,budget,n_imp,kbit,sink,recent,anchor", [
    (2, 8, 150, 60, 20, 0, 4, 16, "alternating"),
    (1, 8, 672, 168, 96, 0, 32, 8, "random"),       # initial + middle + recent, as in Table 1's layout
    (2, 5, 90, 50, 10, 30, 7, 0, "mean"),           # sink only; kbit > half of the middle
    (1, 4, 64, 30, 0, 0, 0, 9, "alternating"),      # recent only, nothing important
    (1, 3, 40, 40, 5, 0, 10, 10, "random"),         # budget == S: identity
    (1, 3, 40, 12, 0, 0, 5, 7, "alternating"),      # budget == protected: the middle is dropped
    (1, 3, 20, 20, 0, 0, 12, 8, "alternating"),     # no middle at all
])
def test_protected_ends_match_brute_force_on_the_middle(oracle, B, Hs, S, budget, n_imp, kbit, sink, recent, anchor):
    """Tokens at the two ends are always kept; the middle is compressed as a
    sequence of its own (independent Python implementation on the sliced scores)."""
    sc = inputs.make_scores(B, Hs, S, seed=S + sink, ties=True)
    idx, kind, bw = oracle.select(sc, budget, n_imp, kbit, anchor, anchor_seed=9, n_sink=sink, n_recent=recent)
    Sm, Bm = S - sink - recent, budget - sink - recent
    W = (Hs + 63) // 64
    for b in range(B):
        def anchor_fn(bits, important):
            if anchor == "alternating":
                return alternating(Hs)
            if anchor == "random":
                z = oracle.splitmix64(9 + b, W)
                return sum(z[w] << (64 * w) for w in range(W)) & ((1 << Hs) - 1)
            disc = [t for t in range(Sm) if t not in important]
            return sum(1 << r for r in range(Hs) if 2 * sum((bits[t] >> r) & 1 for t in disc) > len(disc))
        got_idx, got_kind = idx[b].tolist(), kind[b].tolist()
        want_idx = list(range(sink))
        want_kind = [2] * sink
        want_bits = [0] * S
        if Sm > 0:
            mid = sc[b, :, sink:S - recent].tolist()
            m_idx, m_kind, m_bits = py_select(mid, Bm, n_imp, kbit or Bm, anchor_fn)
            want_idx += [u + sink for u in m_idx]
            want_kind += m_kind
            want_bits[sink:S - recent] = m_bits
        want_idx += list(range(S - recent, S))
        want_kind += [2] * recent
        assert got_idx == want_idx and got_kind == want_kind
        assert [words_to_int(bw[b, t]) for t in range(S)] == want_bits
        assert len(got_idx) == budget and all(x < y for x, y in zip(got_idx, got_idx[1:]))
    # no protected tokens: the plain selection, bit for bit
    plain = oracle.select(sc, budget, min(n_imp, budget), 0, anchor, anchor_seed=9)
    same = oracle.select(sc, budget, min(n_imp, budget), 0, anchor, anchor_seed=9, n_sink=0, n_recent=0)
    assert all(torch.equal(x, y) for x, y in zip(plain, same))


def test_protected_ends_reject_inconsistent_arguments(oracle):
    sc = inputs.make_scores(1, 4, 50, seed=3)
    for kw in (dict(n_sink=20, n_recent=20), dict(n_sink=-1), dict(n_sink=5, n_recent=5, n_important=25)):
        n_imp = kw.pop("n_important", 5)
        with pytest.raises(RuntimeError):
            oracle.select(sc, 30, n_imp, 0, "alternating", **kw)


# ---------------------------------------------------------------- chunk / page level
def py_select_units(sc, unit, budget, n_imp, kbit, anchor_fn):
    """Independent page-level selection: big-int page vectors, pairwise-Hamming medoids."""
    Hs, S = len(sc), len(sc[0])
    tok_bits = [0] * S
    for r in range(Hs):
        for t in py_topk(sc[r], kbit):
            tok_bits[t] |= 1 << r
    tok_imp = []
    for t in range(S):
        acc = np.float32(0.0)
        for r in range(Hs):
            acc = np.float32(acc + np.float32(sc[r][t]))
        tok_imp.append(acc)
    Nu = S // unit
    page_bits, page_imp = [], []
    for u in range(Nu):
        v, acc = 0, np.float32(0.0)
        for j in range(unit):
            v |= tok_bits[u * unit + j] << (j * Hs)       # concatenation, token by token
            acc = np.float32(acc + tok_imp[u * unit + j])
        page_bits.append(v)
        page_imp.append(float(acc))
    important = set(py_topk(page_imp, n_imp // unit))
    anchor = anchor_fn(page_bits, important)
    reps, _ = py_group(page_bits, important, (budget - n_imp) // unit, anchor)
    pages = sorted(important | set(reps))
    idx = [u * unit + j for u in pages for j in range(unit)]
    kind = [1 if u in reps else 0 for u in pages for _ in range(unit)]
    return idx, kind, page_bits


@pytest.mark.parametrize("B,Hs,S,unit,budget,n_imp,kbit,sink,recent,anchor", [
    (2, 4, 96, 8, 32, 16, 0, 0, 0, "alternating"),       # chunks of 8 tokens
    (1, 8, 256, 16, 96, 64, 0, 0, 0, "random"),          # 128-bit page vectors
    (1, 8, 672 + 32, 32, 672, 384, 0, 32, 128, "random"),  # page size 32 with protected ends (Table 1's layout)
    (2, 3, 90, 5, 40, 10, 50, 0, 0, "mean"),             # odd sizes; kbit > half: the mean anchor has one-bits
    (1, 32, 128, 32, 64, 32, 0, 0, 0, "alternating"),    # 1024-bit page vectors
    (1, 4, 64, 4, 64, 16, 0, 0, 0, "mean"),              # budget == S
    (1, 4, 64, 4, 24, 0, 0, 4, 4, "alternating"),        # nothing important
    (1, 4, 64, 4, 24, 24, 0, 0, 0, "alternating"),       # no representatives: paged top-k baseline
])
def test_unit_level_selection_matches_brute_force(oracle, B, Hs, S, unit, budget, n_imp, kbit, sink, recent, anchor):
    sc = inputs.make_scores(B, Hs, S, seed=S + unit, ties=True)
    idx, kind, ub = oracle.select_units(sc, unit, budget, n_imp, kbit, anchor, anchor_seed=4, n_sink=sink,
                                        n_recent=recent)
    Sm, Bm = S - sink - recent, budget - sink - recent
    Hu = Hs * unit
    Wu = (Hu + 63) // 64
    for b in range(B):
        def anchor_fn(bits, important):
            if anchor == "alternating":
                return alternating(Hu)
            if anchor == "random":
                z = oracle.splitmix64(4 + b, Wu)
                return sum(z[w] << (64 * w) for w in range(Wu)) & ((1 << Hu) - 1)
            disc = [u for u in range(len(bits)) if u not in important]
            return sum(1 << r for r in range(Hu) if 2 * sum((bits[u] >> r) & 1 for u in disc) > len(disc))
        mid = sc[b, :, sink:S - recent].tolist()
        m_idx, m_kind, m_bits = py_select_units(mid, unit, Bm, n_imp, kbit or Bm, anchor_fn)
        want_idx = list(range(sink)) + [t + sink for t in m_idx] + list(range(S - recent, S))
        want_kind = [2] * sink + m_kind + [2] * recent
        assert idx[b].tolist() == want_idx and kind[b].tolist() == want_kind
        assert [words_to_int(ub[b, u]) for u in range(Sm // unit)] == m_bits
        # whole units only
        kept = idx[b, sink:budget - recent].view(-1, unit)
        assert ((kept[:, 0] - sink) % unit == 0).all() and (kept[:, 1:] - kept[:, :-1] == 1).all()


def test_unit_of_one_token_is_the_token_level_selection(oracle):
    sc = inputs.make_scores(2, 8, 200, seed=8, ties=True)
    for kw in (dict(), dict(n_sink=3, n_recent=10)):
        a = oracle.select(sc, 60, 30, 0, "mean", 2, **kw)
        b = oracle.select_units(sc, 1, 60, 30, 0, "mean", 2, **kw)
        assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
        mid = a[2][:, kw.get("n_sink", 0):200 - kw.get("n_recent", 0)]
        assert torch.equal(mid, b[2])


def test_unit_level_hand_worked_example(oracle):
    """Two heads, pages of two tokens, eight tokens, per-head top-3.
    head 0 = 9 8 .5 .25 1 0 5 .125 -> top-3 tokens {0, 1, 6};  head 1 = 8 .5 .5 .75 4 6 1 .375 -> {0, 5, 4}.
    Token vectors (bit 0 = head 0): 3 1 0 0 2 2 1 0.  Page vectors (bit 2j + r): page 0 = 0111b,
    page 1 = 0000b, page 2 = 1010b, page 3 = 0001b.  Page importance 17 + 8.5, 1 + 1, 5 + 6, 6 + .5:
    page 0 is the one important page.  Alternating anchor 1010b: distances of pages 1, 2, 3 are 2, 0, 3,
    so the order is 2, 1, 3; two buckets {2} and {1, 3}; in {1, 3} both members cost 1 and the lower
    index wins: representatives 2 and 1.  Kept: pages 0, 1, 2 = tokens 0..5."""
    sc = torch.tensor([[[9.0, 8.0, 0.5, 0.25, 1.0, 0.0, 5.0, 0.125],
                        [8.0, 0.5, 0.5, 0.75, 4.0, 6.0, 1.0, 0.375]]])
    _, _, tb = oracle.select(sc, 3, 3, 3, "alternating")
    assert [int(x) for x in tb[0, :, 0].tolist()] == [3, 1, 0, 0, 2, 2, 1, 0]
    idx, kind, ub = oracle.select_units(sc, 2, 6, 2, 3, "alternating")
    assert [int(x) for x in ub[0, :, 0].tolist()] == [0b0111, 0b0000, 0b1010, 0b0001]
    assert idx.tolist() == [[0, 1, 2, 3, 4, 5]] and kind.tolist() == [[0, 0, 1, 1, 1, 1]]
    # with three buckets every grouped page is its own representative; with one, the medoid of
    # {2, 1, 3} (pairwise distances 2-1: 2, 2-3: 3, 1-3: 1 -> costs 5, 3, 4) is page 1
    idx1, kind1, _ = oracle.select_units(sc, 2, 4, 2, 3, "alternating")
    assert idx1.tolist() == [[0, 1, 2, 3]] and kind1.tolist() == [[0, 0, 1, 1]]


def test_equal_bit_vectors_give_the_first_token_of_each_rank_range(oracle):
    """All grouped tokens alike: every distance and every cost ties, so each bucket's
    representative is its lowest token, i.e. the first of its rank range."""
    S, Hs, Br = 23, 6, 5
    bw = torch.full((S, 1), 0b101101, dtype=torch.int64)
    imp = torch.zeros(S, dtype=torch.uint8)
    imp[[0, 7, 8]] = 1
    disc = [t for t in range(S) if t not in (0, 7, 8)]
    N = len(disc)
    for anchor in ("alternating", "mean", "random"):
        reps, _ = oracle.group(Hs, bw, imp, Br, anchor=anchor, anchor_seed=3)
        assert reps.tolist() == [disc[j * N // Br] for j in range(Br)]
