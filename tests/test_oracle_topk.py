"""Pins for the oracle's top-k + static merge (uniform top-k budget of
Sec. 4.1.2 united with the A-shape static pattern of Sec. 4.1.1): a full
Python sort as brute force, row invariants, tie and special-value cases, and a
hand-worked fixture."""
import math
import os

import numpy as np
import pytest
import torch

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def brute_force_row(srow, i, ns, nl, k):
    """Independent definition: full sort of the non-static causal candidates."""
    static = {j for j in range(0, i + 1) if j < ns or j >= i - nl + 1}
    cand = [j for j in range(0, i + 1) if j not in static]

    def key(j):
        s = float(srow[j])
        if math.isnan(s):
            return (1, 0.0, j)
        return (0, -s if s != 0 else 0.0, j)     # -0.0 and +0.0 tie

    chosen = sorted(cand, key=key)[:k]
    return sorted(static | set(chosen))


def check_rows(sp, idx, cnt, ns, nl, k):
    B, H, NB, _ = sp.shape
    T = idx.shape[-1]
    assert T == min(NB, ns + nl + k)
    for b in range(B):
        for h in range(H):
            for i in range(NB):
                c = int(cnt[b, h, i])
                row = idx[b, h, i].tolist()
                want = brute_force_row(sp[b, h, i].numpy(), i, ns, nl, k)
                assert row[:c] == want, (b, h, i)
                assert all(x == -1 for x in row[c:])
                # invariants
                assert c == min(i + 1, ns + nl + k)
                assert row[c - 1] == i
                assert all(row[a] < row[a + 1] for a in range(c - 1))
                assert all(j in row[:c] for j in range(min(ns, i + 1)))
                assert all(j in row[:c] for j in range(max(0, i - nl + 1), i + 1))


@pytest.mark.parametrize("ns,nl,k", [(1, 2, 2), (0, 1, 3), (2, 3, 0), (1, 1, 40), (3, 4, 5)])
def test_topk_vs_full_sort(oracle, ns, nl, k):
    g = torch.Generator().manual_seed(10 * ns + nl + 100 * k)
    NB = 19
    sp = torch.randn((2, 3, NB, NB), generator=g)
    idx, cnt = oracle.topk(sp, ns, nl, k)
    check_rows(sp, idx, cnt, ns, nl, k)


def test_topk_ties_pick_lowest_index(oracle):
    NB = 12
    sp = torch.zeros((1, 1, NB, NB))
    idx, cnt = oracle.topk(sp, 1, 2, 3)
    # row 10: static {0} U {9,10}; candidates 1..8 all equal -> 1,2,3
    assert idx[0, 0, 10].tolist() == [0, 1, 2, 3, 9, 10]
    check_rows(sp, idx, cnt, 1, 2, 3)
    # few distinct values
    g = torch.Generator().manual_seed(5)
    spq = torch.randint(0, 3, (1, 2, NB, NB), generator=g).float()
    idx, cnt = oracle.topk(spq, 1, 2, 3)
    check_rows(spq, idx, cnt, 1, 2, 3)


def test_topk_special_values(oracle):
    NB = 10
    sp = torch.zeros((1, 1, NB, NB))
    row = torch.tensor([0.0, float("nan"), -0.0, float("-inf"), 0.0, float("inf"), float("nan"), -1.0, 0.0, 0.0])
    sp[0, 0, 9] = row
    idx, cnt = oracle.topk(sp, 1, 1, 4)
    # static {0, 9}; candidates 1..8 ranked: inf(5), then -0.0(2) == 0.0(4) == 0.0(8) by index,
    # then -1(7), -inf(3), NaN(1), NaN(6)
    assert idx[0, 0, 9].tolist() == [0, 2, 4, 5, 8, 9]
    idx, cnt = oracle.topk(sp, 1, 1, 7)
    assert idx[0, 0, 9].tolist() == [0, 1, 2, 3, 4, 5, 7, 8, 9]   # the first NaN beats the second
    check_rows(sp, idx, cnt, 1, 1, 7)


def test_topk_budget_edges(oracle):
    g = torch.Generator().manual_seed(7)
    NB = 9
    sp = torch.randn((1, 2, NB, NB), generator=g)
    idx, cnt = oracle.topk(sp, 1, 2, 0)          # k = 0: the pure A-shape
    for i in range(NB):
        want = sorted({0} | set(range(max(0, i - 1), i + 1)))
        assert idx[0, 0, i, : cnt[0, 0, i]].tolist() == want
    idx, cnt = oracle.topk(sp, 1, 2, NB)         # k >= NB: every causal block
    assert idx.shape[-1] == NB
    for i in range(NB):
        assert idx[0, 1, i, : cnt[0, 1, i]].tolist() == list(range(i + 1))


def test_topk_scale_invariance(oracle):
    g = torch.Generator().manual_seed(8)
    sp = torch.randn((1, 2, 17, 17), generator=g)
    a = oracle.topk(sp, 1, 2, 4)
    b = oracle.topk(sp * 8.0, 1, 2, 4)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


def test_topk_hand_worked_fixture(oracle):
    """tests/golden/topk_hand_worked.txt: a 6-block example ranked by hand."""
    rows, want = [], []
    with open(os.path.join(GOLDEN, "topk_hand_worked.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            left, right = line.split("->")
            rows.append([float(x) for x in left.split()])
            want.append([int(x) for x in right.split()])
    NB = len(rows)
    sp = torch.tensor(rows, dtype=torch.float32).reshape(1, 1, NB, NB)
    idx, cnt = oracle.topk(sp, 1, 2, 2)
    for i in range(NB):
        assert idx[0, 0, i, : cnt[0, 0, i]].tolist() == want[i]


# ---- position-dependent budget (Token Position-Decay, Sec. 4.1.2, Fig. "Stem" (b)) ----

def _decaying(NB, k_first, k_last):
    return torch.tensor([round(k_first + (k_last - k_first) * i / max(NB - 1, 1)) for i in range(NB)],
                        dtype=torch.int32)


def test_tpd_constant_schedule_equals_uniform(oracle):
    g = torch.Generator().manual_seed(5)
    NB, ns, nl, k = 23, 1, 2, 4
    sp = torch.randn((1, 2, NB, NB), generator=g)
    idx_u, cnt_u = oracle.topk(sp, ns, nl, k)
    idx_c, cnt_c = oracle.topk(sp, ns, nl, k, torch.full((NB,), k, dtype=torch.int32))
    assert torch.equal(idx_u, idx_c) and torch.equal(cnt_u, cnt_c)


@pytest.mark.parametrize("ns,nl,k_first,k_last", [(1, 2, 9, 1), (0, 1, 6, 0), (2, 3, 12, 4)])
def test_tpd_vs_full_sort_per_row(oracle, ns, nl, k_first, k_last):
    g = torch.Generator().manual_seed(17 + k_first)
    NB = 29
    sp = torch.randn((2, 2, NB, NB), generator=g)
    kr = _decaying(NB, k_first, k_last)
    k_max = int(kr.max())
    idx, cnt = oracle.topk(sp, ns, nl, k_max, kr)
    assert idx.shape[-1] == min(NB, ns + nl + k_max)
    for b in range(2):
        for h in range(2):
            for i in range(NB):
                c = int(cnt[b, h, i])
                want = brute_force_row(sp[b, h, i].numpy(), i, ns, nl, int(kr[i]))
                assert idx[b, h, i, :c].tolist() == want, (b, h, i)
                assert c == min(i + 1, ns + nl + int(kr[i]))
                assert all(x == -1 for x in idx[b, h, i, c:].tolist())


def test_tpd_budget_is_clamped_to_zero_and_to_the_stated_maximum(oracle):
    g = torch.Generator().manual_seed(3)
    NB, ns, nl, k = 17, 1, 2, 3
    sp = torch.randn((1, 1, NB, NB), generator=g)
    kr = torch.tensor([(-2 if i % 3 == 0 else (100 if i % 3 == 1 else 2)) for i in range(NB)], dtype=torch.int32)
    idx, cnt = oracle.topk(sp, ns, nl, k, kr)
    eff = kr.clamp(0, k)
    for i in range(NB):
        c = int(cnt[0, 0, i])
        assert c == min(i + 1, ns + nl + int(eff[i]))
        assert idx[0, 0, i, :c].tolist() == brute_force_row(sp[0, 0, i].numpy(), i, ns, nl, int(eff[i]))


def test_tpd_lists_are_nested_in_the_budget(oracle):
    """Top-k sets grow monotonically with k: a row's list under budget k_i is a subset of its
    list under any larger budget, and the zero budget leaves exactly the static A-shape."""
    g = torch.Generator().manual_seed(8)
    NB, ns, nl = 21, 1, 3
    sp = torch.randn((1, 2, NB, NB), generator=g)
    small = _decaying(NB, 5, 1)
    big = small + 3
    idx_s, cnt_s = oracle.topk(sp, ns, nl, 8, small)
    idx_b, cnt_b = oracle.topk(sp, ns, nl, 8, big)
    idx_0, cnt_0 = oracle.topk(sp, ns, nl, 8, torch.zeros(NB, dtype=torch.int32))
    for h in range(2):
        for i in range(NB):
            s = set(idx_s[0, h, i, :cnt_s[0, h, i]].tolist())
            b = set(idx_b[0, h, i, :cnt_b[0, h, i]].tolist())
            z = set(idx_0[0, h, i, :cnt_0[0, h, i]].tolist())
            static = {j for j in range(i + 1) if j < ns or j >= i - nl + 1}
            assert z == static and z <= s <= b


# ---- further static patterns of the library (Sec. 4.1.1: Strided, Tri-shape) ----

def _static_set(i, NB, ns, nl, stride, n_dense, reach=0):
    """The definition written out independently of the oracle."""
    if i >= NB - n_dense:
        return set(range(i + 1))
    s = {j for j in range(i + 1) if j < ns or j >= i - nl + 1}
    if stride > 0:
        s |= {j for j in range(i, -1, -stride) if reach == 0 or i - j < reach}
    return s


@pytest.mark.parametrize("stride,reach", [(3, 10), (2, 2), (4, 100), (5, 11), (1, 6)])
def test_dilated_window_vs_definition(oracle, stride, reach):
    g = torch.Generator().manual_seed(stride * 10 + reach)
    NB, ns, nl, k = 31, 1, 2, 3
    sp = torch.randn((1, 2, NB, NB), generator=g)
    idx, cnt = oracle.topk(sp, ns, nl, k, stride=stride, reach=reach)
    assert idx.shape[-1] == min(NB, ns + nl + k + min(NB - 1, reach - 1) // stride)
    for h in range(2):
        for i in range(NB):
            static = _static_set(i, NB, ns, nl, stride, 0, reach)
            cand = [j for j in range(i + 1) if j not in static]
            chosen = sorted(cand, key=lambda j: (-float(sp[0, h, i, j]), j))[:k]
            c = int(cnt[0, h, i])
            assert idx[0, h, i, :c].tolist() == sorted(static | set(chosen)), (h, i)


@pytest.mark.parametrize("ns,nl,k,stride,n_dense", [(1, 2, 3, 4, 0), (0, 1, 2, 3, 0), (1, 2, 3, 0, 3), (2, 2, 4, 5, 2),
                                                   (1, 1, 0, 2, 0), (1, 3, 2, 1, 0)])
def test_strided_and_trishape_vs_definition(oracle, ns, nl, k, stride, n_dense):
    g = torch.Generator().manual_seed(7 * stride + n_dense + k)
    NB = 26
    sp = torch.randn((1, 2, NB, NB), generator=g)
    idx, cnt = oracle.topk(sp, ns, nl, k, stride=stride, n_dense=n_dense)
    T = idx.shape[-1]
    assert T == (NB if n_dense > 0 else min(NB, ns + nl + k + ((NB - 1) // stride if stride else 0)))
    for h in range(2):
        for i in range(NB):
            static = _static_set(i, NB, ns, nl, stride, n_dense)
            cand = [j for j in range(i + 1) if j not in static]
            chosen = sorted(cand, key=lambda j: (-float(sp[0, h, i, j]), j))[:k]
            want = sorted(static | set(chosen))
            c = int(cnt[0, h, i])
            assert c == len(want) <= T
            assert idx[0, h, i, :c].tolist() == want, (h, i)
            assert all(x == -1 for x in idx[0, h, i, c:].tolist())
    # stride 1 makes every causal block static: dense causal lists; so does a strip covering all rows
    if stride == 1:
        assert all(int(cnt[0, 0, i]) == i + 1 for i in range(NB))


def test_trishape_strip_rows_are_dense_and_the_rest_is_the_a_shape(oracle):
    g = torch.Generator().manual_seed(2)
    NB, ns, nl, k, n_dense = 20, 1, 2, 3, 4
    sp = torch.randn((1, 1, NB, NB), generator=g)
    idx_t, cnt_t = oracle.topk(sp, ns, nl, k, n_dense=n_dense)
    idx_a, cnt_a = oracle.topk(sp, ns, nl, k)
    Ta = idx_a.shape[-1]
    for i in range(NB):
        if i >= NB - n_dense:
            assert idx_t[0, 0, i, : i + 1].tolist() == list(range(i + 1)) and int(cnt_t[0, 0, i]) == i + 1
        else:
            assert int(cnt_t[0, 0, i]) == int(cnt_a[0, 0, i])
            assert idx_t[0, 0, i, :Ta].tolist() == idx_a[0, 0, i].tolist()


# ---- per-head configuration (Sec. 4.1.1: settings applied to specific heads) ----

def test_head_pattern_equals_per_head_uniform_calls(oracle):
    g = torch.Generator().manual_seed(12)
    NB, Hq = 22, 4
    sp = torch.randn((2, Hq, NB, NB), generator=g)
    hp = torch.tensor([[1, 2, 5], [0, 1, 0], [2, 3, 2], [9, 9, 9]], dtype=torch.int32)   # last row: clamped to the maxima
    ns, nl, k = 2, 3, 5
    idx, cnt = oracle.topk(sp, ns, nl, k, head_pattern=hp)
    T = idx.shape[-1]
    assert T == min(NB, ns + nl + k)
    eff = [(1, 2, 5), (0, 1, 0), (2, 3, 2), (2, 3, 5)]
    for h, (a, b, c) in enumerate(eff):
        i1, c1 = oracle.topk(sp[:, h:h + 1].contiguous(), a, b, c)
        T1 = i1.shape[-1]
        assert torch.equal(cnt[:, h], c1[:, 0])
        assert torch.equal(idx[:, h, :, :T1], i1[:, 0])
        assert (idx[:, h, :, T1:] == -1).all()


def test_head_pattern_caps_the_budget_schedule(oracle):
    g = torch.Generator().manual_seed(13)
    NB, Hq, ns, nl, k = 18, 2, 1, 2, 6
    sp = torch.randn((1, Hq, NB, NB), generator=g)
    kr = _decaying(NB, 6, 1)
    hp = torch.tensor([[1, 2, 6], [1, 2, 3]], dtype=torch.int32)
    idx, cnt = oracle.topk(sp, ns, nl, k, kr, head_pattern=hp)
    for h, kh in enumerate((6, 3)):
        for i in range(NB):
            want = brute_force_row(sp[0, h, i].numpy(), i, ns, nl, min(int(kr[i]), kh))
            assert idx[0, h, i, : cnt[0, h, i]].tolist() == want
