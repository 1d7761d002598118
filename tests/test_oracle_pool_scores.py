"""Pins for the oracle's pooling and pooled-score steps (pattern computation,
Sec. 4.1.1): closed forms, an independent numpy fp64 evaluation, the GQA head
mapping, linearity and exact power-of-two scaling."""
import numpy as np
import torch


def _rand_bf16(shape, seed):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(shape, generator=g).to(torch.bfloat16)


def test_pool_constant_rows(oracle):
    c = torch.linspace(-2, 2, 16).to(torch.bfloat16)
    x = c.expand(1, 2, 32, 16).contiguous()
    xp = oracle.pool(x, 8)
    assert xp.shape == (1, 2, 4, 16)
    assert torch.equal(xp, c.float().expand(1, 2, 4, 16))


def test_pool_one_hot_token(oracle):
    x = torch.zeros((1, 1, 24, 8), dtype=torch.bfloat16)
    x[0, 0, 13, 5] = 3.0          # block 1 (tokens 8..15) with Bs = 8
    xp = oracle.pool(x, 8)
    want = torch.zeros((1, 1, 3, 8))
    want[0, 0, 1, 5] = 3.0 / 8.0
    assert torch.equal(xp, want)


def test_pool_matches_numpy_mean(oracle):
    x = _rand_bf16((2, 3, 96, 20), 1)
    xp = oracle.pool(x, 32)
    ref = x.double().numpy().reshape(2, 3, 3, 32, 20).mean(axis=3)
    np.testing.assert_allclose(xp.numpy(), ref, rtol=0, atol=2e-7)
    # block order / head order: a transposed reshape would not survive this
    assert abs(xp[1, 2, 0, 7].item() - x[1, 2, :32, 7].double().mean().item()) < 2e-7


def test_scores_match_einsum_and_gqa_mapping(oracle):
    g = torch.Generator().manual_seed(2)
    B, Hq, Hkv, NB, D = 2, 6, 3, 7, 24
    qp = torch.randn((B, Hq, NB, D), generator=g)
    kp = torch.randn((B, Hkv, NB, D), generator=g)
    scale = 0.37
    sp = oracle.scores(qp, kp, scale)
    kexp = kp.repeat_interleave(Hq // Hkv, dim=1)     # head h reads KV head h // G
    ref = np.einsum("bhid,bhjd->bhij", qp.double().numpy(), kexp.double().numpy()) * float(np.float32(scale))
    tri = np.tril(np.ones((NB, NB), dtype=bool))
    np.testing.assert_allclose(sp.numpy()[..., tri], ref[..., tri], rtol=1e-6, atol=1e-6)
    assert np.all(np.isneginf(sp.numpy()[..., ~tri]))


def test_scores_linearity_and_pow2_exact(oracle):
    g = torch.Generator().manual_seed(3)
    qp = torch.randn((1, 2, 5, 16), generator=g)
    kp = torch.randn((1, 1, 5, 16), generator=g)
    s1 = oracle.scores(qp, kp, 0.25)
    s4 = oracle.scores(4.0 * qp, kp, 0.25)
    tri = torch.tril(torch.ones(5, 5, dtype=torch.bool))
    assert torch.equal(s4[..., tri], 4.0 * s1[..., tri])      # power of two: exact
    s3 = oracle.scores(3.0 * qp, kp, 0.25)
    torch.testing.assert_close(s3[..., tri], 3.0 * s1[..., tri], rtol=1e-6, atol=1e-6)


def test_scores_single_dim_hand_values(oracle):
    # D = 1: score(i, j) = scale * qp_i * kp_j, worked by hand.
    qp = torch.tensor([1.0, 2.0, -4.0]).reshape(1, 1, 3, 1)
    kp = torch.tensor([0.5, -1.0, 8.0]).reshape(1, 1, 3, 1)
    sp = oracle.scores(qp, kp, 0.5)
    ninf = float("-inf")
    want = torch.tensor([[0.25, ninf, ninf], [0.5, -1.0, ninf], [-1.0, 2.0, -16.0]])
    assert torch.equal(sp[0, 0], want)


def test_group_shared_scores_are_the_mean_of_the_heads_scores(oracle):
    """Linearity: the score of the group-mean pooled query is the mean of the heads' scores, so
    ranking a KV group by it is ranking by the summed pooled attention of its heads."""
    B, Hq, Hkv, NB, Bs, D = 2, 6, 2, 9, 8, 16
    g = torch.Generator().manual_seed(21)
    q = torch.randn((B, Hq, NB * Bs, D), generator=g).to(torch.bfloat16)
    k = torch.randn((B, Hkv, NB * Bs, D), generator=g).to(torch.bfloat16)
    idx_g, cnt_g, sp_g, qp_g, _ = oracle.select(q, k, Bs, 1, 2, 2, group_shared=True)
    _, _, sp, qp, _ = oracle.select(q, k, Bs, 1, 2, 2)
    assert sp_g.shape == (B, Hkv, NB, NB) and idx_g.shape[1] == Hkv
    want = sp.view(B, Hkv, Hq // Hkv, NB, NB).double().mean(2)
    tri = torch.tril(torch.ones(NB, NB, dtype=torch.bool))
    np.testing.assert_allclose(sp_g[..., tri].numpy(), want[..., tri].numpy(), rtol=1e-5, atol=1e-6)
    np.testing.assert_allclose(qp_g.numpy(), qp.view(B, Hkv, 3, NB, D).double().mean(2).numpy(), rtol=1e-6, atol=1e-7)
    # one head per group: nothing changes
    i1, c1, s1, *_ = oracle.select(q[:, :2], k, Bs, 1, 2, 2, group_shared=True)
    i0, c0, s0, *_ = oracle.select(q[:, :2], k, Bs, 1, 2, 2)
    assert torch.equal(i1, i0) and torch.equal(c1, c0) and torch.equal(s1, s0)
