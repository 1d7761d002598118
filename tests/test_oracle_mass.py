"""Pins for the oracle's cumulative-mass budget (the rule of the FlexPrefill family, which
Sec. 4.1.1 lists among the dynamic algorithms of the framework; no formula in the paper).
Reading: a row takes candidates in ranking order until the selected blocks, static ones included,
hold the fraction gamma of the row's block-level softmax mass; the mass is defined through integer
weights W ~ 2^19 exp(score - max).  Pinned here against numpy fp64 softmax (weights, sufficiency and
minimality of every row), closed forms for equal scores, the limits gamma -> 0 and 1, nesting in
gamma, special values, and a hand-worked fixture."""
import math
import os

import numpy as np
import pytest
import torch

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
ONE = 1 << 19


def _static(i, ns, nl):
    return {j for j in range(i + 1) if j < ns or j >= i - nl + 1}


def test_weights_match_exp_in_fp64(oracle):
    g = torch.Generator().manual_seed(5)
    sp = torch.randn((2, 3, 50, 50), generator=g) * 4.0
    W = oracle.mass_weights(sp).numpy()
    x = sp.double().numpy()
    for i in (0, 1, 17, 49):
        row = x[:, :, i, :i + 1]
        ref = np.exp(row - row.max(-1, keepdims=True))
        got = W[:, :, i, :i + 1] / ONE
        # rounding to a multiple of 2^-19 plus the polynomial's 1.3e-7 relative error
        assert np.abs(got - ref).max() <= 0.5 / ONE + 3e-7
        assert (W[:, :, i, i + 1:] == 0).all()              # beyond the causal limit
        assert (W[:, :, i, :i + 1].max(-1) == ONE).all()    # the maximum weighs exactly 2^19


def test_weights_on_a_dense_grid_against_fp64_exp(oracle):
    """Every weight on a dense grid of differences d = x - m in [-28.5, 0] (200 000 points, plus the
    points around the cut-off and exact ties) against floor(2^19 e^d + 1/2) evaluated in fp64.
    Stated bound: |W - 2^19 e^d| <= 0.5 (rounding to an integer) + 0.2 (fp32 evaluation: the
    polynomial's truncation error of 1.3e-7 and about three fp32 roundings of 2^-24, relative to a
    weight of at most 2^19), hence W differs from the fp64 rounding by at most 1 and only where
    2^19 e^d lies within 0.2 of a half-integer.  A wrong coefficient, a dropped term or a wrong
    exponent split breaks the bound; the cut-off is where (x - m) log2 e, rounded to fp32, falls
    below -40; weights never increase as d falls."""
    n_rows, n = 50, 4001
    d = -np.linspace(0.0, 28.5, n_rows * (n - 1))
    # keep the maximum (d = 0) in column 0 of every row; a row is causal in full (KV prefix)
    rows = np.concatenate([np.zeros((n_rows, 1)), d.reshape(n_rows, n - 1)], axis=1).astype(np.float32)
    # an arbitrary common offset must not matter beyond the fp32 subtraction, which is exact here:
    # the grid itself is fp32 and m = 0
    sp = torch.from_numpy(rows).reshape(1, n_rows, 1, n)
    W = oracle.mass_weights(sp)[0, :, 0].numpy().astype(np.int64)
    x = rows.astype(np.float64)
    exact = np.exp(x) * ONE
    t32 = (rows.astype(np.float32) * np.float32(1.44269504088896340736)).astype(np.float32)
    cut = ~(t32 >= np.float32(-40.0))
    assert cut.any() and (~cut).sum() > 190000
    assert (W[cut] == 0).all()
    live = ~cut
    assert np.abs(W[live] - exact[live]).max() <= 0.7
    ref = np.floor(exact + 0.5).astype(np.int64)
    off = W[live] != ref[live]
    assert np.abs(W[live] - ref[live]).max() <= 1
    frac = exact[live] - np.floor(exact[live])
    assert (np.abs(frac[off] - 0.5) <= 0.2).all()
    assert off.mean() < 0.05
    flat = W[:, 1:].reshape(-1)                            # d falls along the flattened grid
    assert (np.diff(flat) <= 0).all()
    assert (W[:, 0] == ONE).all()
    # ties: equal scores weigh the same whatever their position, and a shifted row (same
    # differences, representable exactly) gives the same weights
    tied = torch.tensor([1.5, -0.25, 1.5, -0.25, -0.25, 1.5, -7.0, -7.0]).reshape(1, 1, 1, 8)
    Wt = oracle.mass_weights(tied)[0, 0, 0].tolist()
    assert Wt[0] == Wt[2] == Wt[5] == ONE and Wt[1] == Wt[3] == Wt[4] and Wt[6] == Wt[7]
    assert oracle.mass_weights(tied + 64.0)[0, 0, 0].tolist() == Wt
    assert Wt[1] == int(math.floor(math.exp(-1.75) * ONE + 0.5)) and Wt[6] == int(math.floor(math.exp(-8.5) * ONE + 0.5))


def test_weights_of_special_values(oracle):
    nan, inf = float("nan"), float("inf")
    sp = torch.tensor([[0.0, -inf, nan, -100.0, -0.0, 1.0, -1.0, 0.5],
                       [-inf, -inf, nan, -inf, -inf, -inf, -inf, -inf],
                       [inf, 3.0, inf, nan, -inf, 0.0, 1.0, 2.0],
                       [nan, nan, nan, nan, nan, nan, nan, nan]]).reshape(1, 4, 1, 8)
    # one query block at the end of 8 key blocks (a KV prefix of 7): the whole row is causal
    W = oracle.mass_weights(sp)[0, :, 0].tolist()
    e = lambda d: int(math.floor(math.exp(d) * ONE + 0.5))
    assert W[0] == [e(-1), 0, 0, 0, e(-1), ONE, e(-2), e(-0.5)]
    assert W[1] == [ONE, ONE, 0, ONE, ONE, ONE, ONE, ONE]     # all -inf: equal to the maximum
    assert W[2] == [ONE, 0, ONE, 0, 0, 0, 0, 0]               # +inf outweighs everything finite
    assert W[3] == [0] * 8


@pytest.mark.parametrize("gamma", [0.3, 0.7, 0.9, 0.95, 0.99])
@pytest.mark.parametrize("ns,nl,k", [(1, 2, 100), (0, 1, 100), (2, 3, 5)])
def test_rows_are_sufficient_and_minimal_in_fp64(oracle, gamma, ns, nl, k):
    """Against an independent fp64 softmax: the selected mass reaches gamma, and without the worst
    ranked dynamic block it would not (unless the count budget cut the row short)."""
    NB = 60
    g = torch.Generator().manual_seed(int(gamma * 100) + ns)
    sp = torch.randn((1, 2, NB, NB), generator=g) * 2.5
    idx, cnt = oracle.topk(sp, ns, nl, k, gamma=gamma)
    g32 = float(np.float32(gamma))
    checked = 0
    for h in range(2):
        for i in range(NB):
            x = sp[0, h, i, :i + 1].double().numpy()
            p = np.exp(x - x.max())
            p /= p.sum()
            sel = idx[0, h, i, :int(cnt[0, h, i])].tolist()
            st = _static(i, ns, nl)
            assert st <= set(sel) and sel == sorted(set(sel)) and sel[-1] == i
            dyn = [j for j in sel if j not in st]
            cand = sorted((j for j in range(i + 1) if j not in st), key=lambda j: (-x[j], j))
            assert sorted(dyn) == sorted(cand[:len(dyn)])          # a prefix of the ranking
            tol = (i + 1) * 1.0 / ONE + 1e-6                        # quantisation of the weights
            mass = p[sel].sum()
            capped = len(dyn) == min(k, len(cand))
            if not capped:
                assert mass >= g32 - tol, (h, i, mass)
            if dyn:
                worst = cand[len(dyn) - 1]
                assert mass - p[worst] < g32 + tol, (h, i)
                checked += 1
    assert checked > 20


def test_gamma_limits_and_nesting(oracle):
    g = torch.Generator().manual_seed(11)
    sp = torch.randn((1, 2, 40, 40), generator=g)
    ns, nl, k = 1, 2, 12
    idx0, cnt0 = oracle.topk(sp, ns, nl, k, gamma=0.0)
    idxa, cnta = oracle.topk(sp, ns, nl, 0)                          # static only
    assert torch.equal(cnt0, cnta) and torch.equal(idx0[..., :idxa.shape[-1]], idxa)
    idx1, cnt1 = oracle.topk(sp, ns, nl, k, gamma=1.0)               # every weight is needed: the count cap binds
    idxc, cntc = oracle.topk(sp, ns, nl, k)
    assert torch.equal(idx1, idxc) and torch.equal(cnt1, cntc)
    prev = None
    for gamma in (0.1, 0.4, 0.6, 0.8, 0.9, 0.97, 1.0):
        idx, cnt = oracle.topk(sp, ns, nl, k, gamma=gamma)
        sets = [[set(idx[0, h, i, :int(cnt[0, h, i])].tolist()) for i in range(40)] for h in range(2)]
        if prev is not None:
            assert all(prev[h][i] <= sets[h][i] for h in range(2) for i in range(40))
        prev = sets


@pytest.mark.parametrize("gamma", [0.25, 0.5, 0.75, 0.9])
def test_equal_scores_closed_form(oracle, gamma):
    """All scores equal: every block weighs 2^19, so a row of n causal blocks needs
    ceil(Gamma n / 65536) blocks in all, static ones first, then the lowest candidate indices."""
    NB, ns, nl, k = 37, 2, 3, 30
    sp = torch.full((1, 1, NB, NB), 0.375)
    idx, cnt = oracle.topk(sp, ns, nl, k, gamma=gamma)
    Gamma = int(math.floor(float(np.float32(gamma)) * 65536 + 0.5))
    for i in range(NB):
        st = _static(i, ns, nl)
        cand = [j for j in range(i + 1) if j not in st]
        need_blocks = -(-(Gamma * (i + 1)) // 65536)
        m = min(max(need_blocks - len(st), 0), k, len(cand))
        want = sorted(st | set(cand[:m]))
        assert idx[0, 0, i, :int(cnt[0, 0, i])].tolist() == want, i


def test_count_budgets_stay_caps(oracle):
    g = torch.Generator().manual_seed(3)
    sp = torch.randn((1, 2, 50, 50), generator=g) * 0.1            # flat rows: the mass budget wants many blocks
    sched = torch.randint(0, 9, (50,), generator=g).to(torch.int32)
    idx, cnt = oracle.topk(sp, 1, 2, 8, k_per_row=sched, gamma=0.99)
    idxc, cntc = oracle.topk(sp, 1, 2, 8, k_per_row=sched)
    assert (cnt <= cntc).all()
    assert torch.equal(cnt[:, :, 30:], cntc[:, :, 30:])            # long flat rows: the schedule binds
    hp = torch.tensor([[1, 2, 3], [0, 1, 8]], dtype=torch.int32)
    idx, cnt = oracle.topk(sp, 1, 2, 8, head_pattern=hp, gamma=0.6)
    idxc, cntc = oracle.topk(sp, 1, 2, 8, head_pattern=hp)
    assert (cnt <= cntc).all() and (cnt[0, 0] <= 3 + 3).all()


def test_hand_worked_fixture(oracle):
    ln2 = math.log(2.0)
    row = torch.tensor([0.0, -1.0, -2.0, -3.0, -1.0, -2.0, 0.0, -5.0], dtype=torch.float64) * ln2
    sp = row.float().reshape(1, 1, 1, 8)                            # one query block after a prefix of 7
    cases = 0
    for line in open(os.path.join(GOLDEN, "mass_budget_hand_worked.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        gamma, want = line.split("->")
        idx, cnt = oracle.topk(sp, 1, 1, 6, gamma=float(gamma))
        assert idx[0, 0, 0, :int(cnt[0, 0, 0])].tolist() == [int(t) for t in want.split()], gamma
        cases += 1
    assert cases == 5
