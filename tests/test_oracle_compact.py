"""Pins for the oracle's compaction (the final cache holds the retained tokens,
Sec. 3.2): rows are byte-copies of the source rows, checked against torch's own
index_select; the paged source must give the same bytes as the dense one."""
import pytest
import torch

from paper_2503_00022_amd import inputs


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_dense_rows_are_byte_equal(oracle, dtype):
    w = inputs.Workload("t", 2, 4, 2, 96, 32, dtype, 24, 0.5, "alternating", True)
    _, k, v = inputs.make_qkv(w, 3)
    g = torch.Generator().manual_seed(1)
    idx = torch.stack([torch.randperm(w.S, generator=g)[: w.budget].sort().values for _ in range(w.B)]).int()
    ko, vo = oracle.compact(k, v, idx)
    for b in range(w.B):
        assert torch.equal(ko[b], k[b].index_select(1, idx[b].long()))
        assert torch.equal(vo[b], v[b].index_select(1, idx[b].long()))


def test_paged_equals_dense(oracle):
    w = inputs.Workload("t", 3, 8, 2, 128, 16, "bf16", 40, 0.25, "alternating", True, paged=True, block_size=16)
    _, k, v = inputs.make_qkv(w, 4)
    bt = inputs.make_block_table(w, 9)
    assert sorted(bt.view(-1).tolist()) == list(range(w.B * w.S // 16))
    kp, vp = inputs.to_paged(k, bt, 16), inputs.to_paged(v, bt, 16)
    # the pool really holds token t of (b, h) where the table says
    b, h, t = 2, 1, 77
    assert torch.equal(kp[bt[b, t // 16], t % 16, h], k[b, h, t])
    g = torch.Generator().manual_seed(2)
    idx = torch.stack([torch.randperm(w.S, generator=g)[: w.budget].sort().values for _ in range(w.B)]).int()
    kd, vd = oracle.compact(k, v, idx)
    ko, vo = oracle.compact(kp, vp, idx, block_table=bt, block_size=16, dense_shape=(w.B, w.Hkv, w.S, w.D))
    assert torch.equal(ko, kd) and torch.equal(vo, vd)


def test_identity_when_budget_is_everything(oracle):
    w = inputs.Workload("t", 1, 2, 2, 20, 8, "f32", 20, 0.5, "alternating", True)
    _, k, v = inputs.make_qkv(w, 5)
    idx = torch.arange(20, dtype=torch.int32)[None]
    ko, vo = oracle.compact(k, v, idx)
    assert torch.equal(ko, k) and torch.equal(vo, v)
