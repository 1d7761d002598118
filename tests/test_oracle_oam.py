"""Pins for the oracle's output-aware ranking score (Stem's Output-Aware Metric, Sec. 4.1.2,
Fig. "Stem" (c)): the value-magnitude pooling against closed forms and numpy, the score against
its definition written with numpy, and the invariances the definition implies for the selection.
The formula itself is a reading (the paper prints none): parity with the paper is unpinned."""
import math

import numpy as np
import torch


def _rand(shape, seed):
    return torch.randn(shape, generator=torch.Generator().manual_seed(seed)).to(torch.bfloat16)


def test_vnorm_closed_forms(oracle):
    Bs, D, NB = 8, 16, 5
    v = torch.zeros((1, 2, NB * Bs, D), dtype=torch.bfloat16)
    v[0, 0] = 0.5                                   # every vector has norm 0.5 * sqrt(D)
    v[0, 1, 3 * Bs + 2, 7] = 3.0                    # one token of block 3 has norm 3, the rest 0
    vn = oracle.vnorm(v, Bs)
    assert vn.shape == (1, 2, NB)
    np.testing.assert_allclose(vn[0, 0].numpy(), 0.5 * math.sqrt(D), rtol=1e-7)
    want = np.zeros(NB, dtype=np.float32)
    want[3] = 3.0 / Bs
    np.testing.assert_array_equal(vn[0, 1].numpy(), want)


def test_vnorm_vs_numpy(oracle):
    Bs, D, NB = 16, 32, 7
    v = _rand((2, 3, NB * Bs, D), 4)
    want = np.linalg.norm(v.double().numpy().reshape(2, 3, NB, Bs, D), axis=-1).mean(-1)
    np.testing.assert_allclose(oracle.vnorm(v, Bs).numpy(), want, rtol=2e-7)


def test_scores_oam_is_score_plus_log_magnitude(oracle):
    B, Hq, Hkv, NB = 2, 4, 2, 9
    g = torch.Generator().manual_seed(6)
    sp = torch.randn((B, Hq, NB, NB), generator=g)
    vn = torch.rand((B, Hkv, NB), generator=g) + 0.1
    vn[0, 1, 4] = 0.0                                # a block of zero values
    got = oracle.scores_oam(sp, vn)
    for b in range(B):
        for h in range(Hq):
            for i in range(NB):
                for j in range(NB):
                    if j > i:
                        assert got[b, h, i, j] == sp[b, h, i, j]
                    elif vn[b, h // 2, j] == 0:
                        assert got[b, h, i, j] == -math.inf
                    else:
                        want = np.float32(np.float64(sp[b, h, i, j]) + np.log(np.float64(vn[b, h // 2, j])))
                        assert got[b, h, i, j].item() == want


def test_selection_ignores_a_common_value_scale_and_follows_value_magnitude(oracle):
    Bs, D, NB, ns, nl, k = 8, 16, 24, 1, 2, 4
    q, kk, v = _rand((1, 2, NB * Bs, D), 1), _rand((1, 1, NB * Bs, D), 2), _rand((1, 1, NB * Bs, D), 3)
    idx, cnt, *_ = oracle.select(q, kk, Bs, ns, nl, k, v=v)
    # V -> 4 V adds ln 4 to every candidate's score (exactly a power of two): same lists
    idx4, cnt4, *_ = oracle.select(q, kk, Bs, ns, nl, k, v=(v.float() * 4).to(torch.bfloat16))
    assert torch.equal(idx, idx4) and torch.equal(cnt, cnt4)
    # values of equal magnitude everywhere: the metric reduces to the plain score
    v_const = torch.ones_like(v)
    idx_c, _, *_ = oracle.select(q, kk, Bs, ns, nl, k, v=v_const)
    idx_p, _, *_ = oracle.select(q, kk, Bs, ns, nl, k)
    assert torch.equal(idx_c, idx_p)
    # blocks whose values vanish are never picked while another candidate is left, and a block with
    # huge values always is
    v2 = v.clone()
    dead, loud = [5, 9, 10], 7
    for j in dead:
        v2[0, 0, j * Bs:(j + 1) * Bs] = 0
    v2[0, 0, loud * Bs:(loud + 1) * Bs] *= 2.0 ** 40
    idx2, cnt2, *_ = oracle.select(q, kk, Bs, ns, nl, k, v=v2)
    for h in range(2):
        for i in range(NB):
            row = idx2[0, h, i, : cnt2[0, h, i]].tolist()
            static = {j for j in range(i + 1) if j < ns or j >= i - nl + 1}
            dyn = [j for j in row if j not in static]
            n_live = len([j for j in range(i + 1) if j not in static and j not in dead])
            if n_live >= k:
                assert not set(dyn) & set(dead), (h, i, row)
            if loud <= i and loud not in static:
                assert loud in dyn, (h, i, row)
