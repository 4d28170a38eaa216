"""Pins of the Top-K and compaction oracles (CPU only): a Python sort under the
stated total order, invariants, crafted ties, signed zeros, NaN, K = 1 and K = N,
byte equality of the gather."""
import math

import numpy as np
import pytest
import torch

import oracle


def _py_topk(row, K):
    def key(i):
        v = row[i]
        if math.isnan(v):
            return (1, 0.0, i)
        return (0, -(v + 0.0), i)          # adding 0.0 folds -0.0 onto +0.0
    return sorted(sorted(range(len(row)), key=key)[:K])


@pytest.mark.parametrize("N,K", [(1, 1), (17, 1), (17, 17), (64, 19), (257, 100)])
def test_topk_matches_python_sort(N, K):
    g = torch.Generator().manual_seed(N * 31 + K)
    s = torch.randn(5, N, generator=g)
    s[1] = torch.round(s[1] * 2) / 2            # many duplicates
    s[2] = 0.25
    if N > 4:
        s[3, ::3] = float("nan")
        s[4, 1] = -0.0; s[4, 2] = 0.0; s[4, 3] = float("inf"); s[4, 4] = float("-inf")
    idx = oracle.topk(s, K)
    assert idx.dtype == torch.int32 and idx.shape == (5, K)
    for r in range(5):
        assert idx[r].tolist() == _py_topk(s[r].tolist(), K)


def test_topk_ties_and_special_values():
    assert oracle.topk(torch.full((1, 9), 3.0), 4)[0].tolist() == [0, 1, 2, 3]
    # duplicates straddling the boundary: lower index wins
    s = torch.tensor([[1.0, 5.0, 2.0, 5.0, 2.0, 2.0, 0.0]])
    assert oracle.topk(s, 3)[0].tolist() == [1, 2, 3]
    assert oracle.topk(s, 4)[0].tolist() == [1, 2, 3, 4]
    # -0.0 and +0.0 tie
    z = torch.tensor([[-1.0, 0.0, -0.0, -0.0, 0.0]])
    assert oracle.topk(z, 2)[0].tolist() == [1, 2]
    z = torch.tensor([[-1.0, -0.0, 0.0, 1.0]])
    assert oracle.topk(z, 2)[0].tolist() == [1, 3]
    # NaN ranks below every number, -inf included
    n = torch.tensor([[float("nan"), float("-inf"), float("nan"), -3.0]])
    assert oracle.topk(n, 2)[0].tolist() == [1, 3]
    assert oracle.topk(n, 3)[0].tolist() == [0, 1, 3]
    with pytest.raises(ValueError):
        oracle.topk(n, 0)
    with pytest.raises(ValueError):
        oracle.topk(n, 5)


def test_topk_invariants_on_random_rows():
    g = torch.Generator().manual_seed(9)
    s = torch.randn(6, 500, generator=g)
    K = 150
    idx = oracle.topk(s, K).to(torch.int64)
    for r in range(6):
        kept = idx[r]
        assert bool((kept[1:] > kept[:-1]).all())
        mask = torch.zeros(500, dtype=torch.bool); mask[kept] = True
        assert float(s[r][mask].min()) >= float(s[r][~mask].max())
        assert int(mask.sum()) == K


def test_compact_is_an_ordered_gather():
    g = torch.Generator().manual_seed(10)
    kv = torch.randn(2, 3, 40, 8, generator=g).to(torch.bfloat16)
    s = torch.randn(6, 40, generator=g)
    idx = oracle.topk(s, 12).view(2, 3, 12)
    out = oracle.compact(kv, idx)
    assert out.shape == (2, 3, 12, 8) and out.dtype == torch.bfloat16
    for l in range(2):
        for h in range(3):
            for j in range(12):
                assert torch.equal(out[l, h, j].view(torch.int16), kv[l, h, int(idx[l, h, j])].view(torch.int16))
    full = oracle.topk(s, 40).view(2, 3, 40)
    assert torch.equal(oracle.compact(kv, full).view(torch.int16), kv.view(torch.int16))
    # order preserved: a cache whose rows hold their own token index comes back ascending
    marker = torch.arange(40, dtype=torch.float32).view(1, 1, 40, 1).expand(2, 3, 40, 8).contiguous()
    got = oracle.compact(marker, idx)[..., 0]
    assert bool((got[..., 1:] > got[..., :-1]).all())


def test_mask_marks_exactly_the_kept_tokens():
    g = torch.Generator().manual_seed(12)
    s = torch.randn(6, 50, generator=g)
    idx = oracle.topk(s, 17).view(2, 3, 17)
    M = oracle.mask(idx, 50)
    assert M.shape == (2, 3, 50) and M.dtype == torch.uint8
    for l in range(2):
        for h in range(3):
            kept = set(idx[l, h].tolist())
            assert [int(v) for v in M[l, h]] == [1 if n in kept else 0 for n in range(50)]
    assert int(M.sum()) == 6 * 17
    # the mask selects the same rows, in the same order, as the gather
    kv = torch.randn(2, 3, 50, 4, generator=g)
    assert torch.equal(kv[M.bool()].view(2, 3, 17, 4), oracle.compact(kv, idx))


def test_topk_pooled_matches_sort_over_pairs():
    """Brute force over (head, token) pairs with Python's sort under the stated order."""
    g = torch.Generator().manual_seed(13)
    L, H, N, K = 3, 4, 23, 5
    s = torch.randn(L, H, N, generator=g)
    s[1] = torch.round(s[1] * 2) / 2          # ties across heads
    s[2, 1] += 3.0                            # one head takes most of the budget
    flat, counts = oracle.topk_pooled(s, K)
    assert flat.shape == (L, H * K) and counts.shape == (L, H) and flat.dtype == torch.int32
    for l in range(L):
        pairs = sorted(((-float(s[l, h, n]), h * N + n) for h in range(H) for n in range(N)))[:H * K]
        want = sorted(p[1] for p in pairs)
        assert flat[l].tolist() == want
        assert counts[l].tolist() == [sum(1 for f in want if f // N == h) for h in range(H)]
        assert int(counts[l].sum()) == H * K
    assert int(counts[2, 1]) > K              # the budget moved to the strong head
    # equal scores everywhere: the lowest flat indices are kept, i.e. head 0 first
    flat, counts = oracle.topk_pooled(torch.zeros(1, 3, 10), 4)
    assert flat[0].tolist() == list(range(12)) and counts[0].tolist() == [10, 2, 0]
