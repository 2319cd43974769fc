"""Pins for the oracle's row layout, mask and position ids (no GPU)."""
import os

import numpy as np
import pytest
import torch

from oracle import tidar_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_q_len_footnote():
    # Section 3.3 footnote: q_len = block_len * (1 + block_len)
    assert [O.q_len(k) for k in (4, 8, 16)] == [20, 72, 272]


def test_mask_worked_example_k3():
    gold = np.loadtxt(os.path.join(GOLD, "decode_mask_k3.txt"), dtype=np.int64)
    for L in (0, 3, 7):     # Figure 3's example uses a prefix of length 3
        M = O.decode_mask(3, L)
        assert M.shape == (12, L + 12)
        assert bool(M[:, :L].all())
        assert np.array_equal(M[:, L:].numpy().astype(np.int64), gold)


@pytest.mark.parametrize("k,count", [(3, 51), (4, 114), (8, 836), (16, 6408)])
def test_mask_closed_form_count(k, count):
    # causal triangle + k*k rows each seeing j drafts + k*k rows each seeing k block mates
    assert k * (k + 1) // 2 + k * k * (k + 1) // 2 + k ** 3 == count
    assert int(O.decode_mask(k, 5)[:, 5:].sum()) == count


@pytest.mark.parametrize("k", [1, 2, 4, 5, 8])
def test_mask_structure(k):
    L = 6
    M = O.decode_mask(k, L)
    R = O.q_len(k)
    new = M[:, L:]
    # causal rows never see a mask column (makes causal logits independent of the mask tokens)
    assert not bool(new[:k, k:].any())
    # causal part is lower triangular with a full diagonal
    assert torch.equal(new[:k, :k], torch.tril(torch.ones(k, k, dtype=torch.bool)))
    # mask rows: block-diagonal over mask columns, full blocks
    blk = torch.arange(k * k) // k
    assert torch.equal(new[k:, k:], blk[:, None] == blk[None, :])
    # block j sees exactly drafts c_1..c_j
    for j in range(1, k + 1):
        for s in range(1, k + 1):
            assert int(new[O.row_of_blk(k, j, s), :k].sum()) == j
            assert bool(new[O.row_of_blk(k, j, s), :j].all())
    assert M.shape == (R, L + R)


def test_k1_is_causal_plus_one_self_attending_mask_row():
    M = O.decode_mask(1, 4)
    assert torch.equal(M[0], torch.tensor([1, 1, 1, 1, 1, 0], dtype=torch.bool))
    assert torch.equal(M[1], torch.tensor([1, 1, 1, 1, 1, 1], dtype=torch.bool))


@pytest.mark.parametrize("k", [1, 3, 4, 16])
def test_positions(k):
    L = 11
    pos = O.decode_positions(k, L)
    for i in range(1, k + 1):
        assert int(pos[O.row_of_c(i)]) == L + i - 1
    for j in range(1, k + 1):
        # Section 4.3.3: the causal output of draft j and the first slot of block j predict the same position.
        # causal rows are label shifted (row at p predicts p+1), mask rows are not (row at p predicts p).
        assert int(pos[O.row_of_blk(k, j, 1)]) == int(pos[O.row_of_c(j)]) + 1
        for s in range(2, k + 1):
            assert int(pos[O.row_of_blk(k, j, s)]) == int(pos[O.row_of_blk(k, j, s - 1)]) + 1


def test_prefill_mask():
    P, k = 5, 3
    M = O.prefill_mask(P, k)
    assert torch.equal(M[:P, :P], torch.tril(torch.ones(P, P, dtype=torch.bool)))
    assert not bool(M[:P, P:].any())
    assert bool(M[P:].all())
    # a decode mask with block a of a step whose drafts were all accepted is this mask's last block:
    # block k of decode_mask(k, L) sees prefix + c_1..c_k + itself  ==  prefill block over P = L + k
    D = O.decode_mask(k, P - k)
    rows = [O.row_of_blk(k, k, s) for s in range(1, k + 1)]
    cols = list(range(P)) + [P - k + O.row_of_blk(k, k, s) for s in range(1, k + 1)]
    assert torch.equal(D[rows][:, cols], M[P:])
    assert int(D[rows].sum()) == int(M[P:].sum())
