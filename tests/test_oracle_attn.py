"""Pins for the oracle's sparse attention step (Sec. 4.1.1: sparse attention
executed on the regions the pattern computation located): equality with dense
causal attention when every block is selected (library routine and numpy
brute force), brute-force masked softmax on tiny inputs, rows summing to one,
log-sum-exp, permutation invariance inside non-diagonal blocks, the block
diagonal special case, a closed form for constant keys and the row-subset
interface."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F


def _qkv(B, Hq, Hkv, S, D, seed):
    g = torch.Generator().manual_seed(seed)
    q = torch.randn((B, Hq, S, D), generator=g).to(torch.bfloat16)
    k = torch.randn((B, Hkv, S, D), generator=g).to(torch.bfloat16)
    v = torch.randn((B, Hkv, S, D), generator=g).to(torch.bfloat16)
    return q, k, v


def _all_causal(B, Hq, NB):
    idx = torch.full((B, Hq, NB, NB), -1, dtype=torch.int32)
    cnt = torch.empty((B, Hq, NB), dtype=torch.int32)
    for i in range(NB):
        idx[:, :, i, : i + 1] = torch.arange(i + 1, dtype=torch.int32)
        cnt[:, :, i] = i + 1
    return idx, cnt


def brute_force(q, k, v, idx, cnt, Bs, scale):
    """Expand the block lists to a dense S x S boolean mask; plain softmax in fp64."""
    B, Hq, S, D = q.shape
    G = Hq // k.shape[1]
    out = np.zeros((B, Hq, S, D))
    lse = np.zeros((B, Hq, S))
    for b in range(B):
        for h in range(Hq):
            qq = q[b, h].double().numpy()
            kk = k[b, h // G].double().numpy()
            vv = v[b, h // G].double().numpy()
            mask = np.zeros((S, S), dtype=bool)
            for i in range(S // Bs):
                for j in idx[b, h, i, : int(cnt[b, h, i])].tolist():
                    mask[i * Bs:(i + 1) * Bs, j * Bs:(j + 1) * Bs] = True
            mask &= np.tril(np.ones((S, S), dtype=bool))
            x = np.where(mask, float(np.float32(scale)) * (qq @ kk.T), -np.inf)
            m = x.max(axis=1, keepdims=True)
            p = np.exp(x - m)
            out[b, h] = (p @ vv) / p.sum(axis=1, keepdims=True)
            lse[b, h] = (m + np.log(p.sum(axis=1, keepdims=True)))[:, 0]
    return out, lse


def test_all_blocks_equals_dense_causal_sdpa(oracle):
    B, Hq, Hkv, S, D, Bs = 2, 4, 2, 64, 16, 8
    q, k, v = _qkv(B, Hq, Hkv, S, D, 0)
    idx, cnt = _all_causal(B, Hq, S // Bs)
    out, lse = oracle.attn(q, k, v, idx, cnt, Bs)
    G = Hq // Hkv
    ref = F.scaled_dot_product_attention(q.float(), k.float().repeat_interleave(G, 1),
                                         v.float().repeat_interleave(G, 1), is_causal=True)
    torch.testing.assert_close(out, ref, rtol=1e-4, atol=2e-5)
    bf, bl = brute_force(q, k, v, idx, cnt, Bs, oracle.default_scale(D))
    np.testing.assert_allclose(out.numpy(), bf, rtol=0, atol=1e-6)
    np.testing.assert_allclose(lse.numpy(), bl, rtol=0, atol=2e-6)


@pytest.mark.parametrize("ns,nl,k,scale", [(1, 2, 2, None), (0, 1, 3, 0.5), (2, 1, 0, None)])
def test_sparse_vs_brute_force_tiny(oracle, ns, nl, k, scale):
    B, Hq, Hkv, S, D, Bs = 1, 4, 2, 48, 8, 4
    q, kk, v = _qkv(B, Hq, Hkv, S, D, 1)
    idx, cnt, *_ = oracle.select(q, kk, Bs, ns, nl, k, scale)
    assert int(cnt.max()) < S // Bs          # really sparse
    out, lse = oracle.attn(q, kk, v, idx, cnt, Bs, scale)
    sc = oracle.default_scale(D) if scale is None else scale
    bf, bl = brute_force(q, kk, v, idx, cnt, Bs, sc)
    np.testing.assert_allclose(out.numpy(), bf, rtol=0, atol=1e-6)
    np.testing.assert_allclose(lse.numpy(), bl, rtol=0, atol=2e-6)


def test_unit_values_give_unit_output(oracle):
    q, k, v = _qkv(1, 2, 1, 32, 8, 2)
    v = torch.ones_like(v)
    idx, cnt, *_ = oracle.select(q, k, 4, 1, 1, 2)
    out, _ = oracle.attn(q, k, v, idx, cnt, 4)
    np.testing.assert_allclose(out.numpy(), 1.0, rtol=0, atol=1e-6)


def test_constant_keys_closed_form(oracle):
    # K == 0 -> every visible selected key gets the same weight, so
    # out_t = mean of v over {s <= t, block(s) selected}; lse_t = log(count).
    S, Bs, D = 24, 4, 2
    q, _, _ = _qkv(1, 1, 1, S, D, 3)
    k = torch.zeros((1, 1, S, D), dtype=torch.bfloat16)
    v = torch.arange(S, dtype=torch.float32).reshape(1, 1, S, 1).expand(1, 1, S, D).to(torch.bfloat16).contiguous()
    NB = S // Bs
    idx = torch.full((1, 1, NB, 2), -1, dtype=torch.int32)
    cnt = torch.empty((1, 1, NB), dtype=torch.int32)
    for i in range(NB):                       # sink block 0 + the diagonal
        sel = sorted({0, i})
        idx[0, 0, i, : len(sel)] = torch.tensor(sel, dtype=torch.int32)
        cnt[0, 0, i] = len(sel)
    out, lse = oracle.attn(q, k, v, idx, cnt, Bs)
    for t in range(S):
        i = t // Bs
        vis = [s for s in range(t + 1) if s // Bs in (0, i)]
        assert abs(out[0, 0, t, 0].item() - np.mean(vis)) < 1e-5
        assert abs(lse[0, 0, t].item() - np.log(len(vis))) < 1e-6


def test_permutation_inside_selected_block(oracle):
    q, k, v = _qkv(1, 1, 1, 32, 8, 4)
    Bs = 8
    idx, cnt = _all_causal(1, 1, 4)
    out0, _ = oracle.attn(q, k, v, idx, cnt, Bs)
    perm = torch.tensor([3, 1, 7, 0, 2, 6, 5, 4])
    k2, v2 = k.clone(), v.clone()
    k2[0, 0, 8:16] = k[0, 0, 8:16][perm]      # shuffle keys+values of block 1
    v2[0, 0, 8:16] = v[0, 0, 8:16][perm]
    out1, _ = oracle.attn(q, k2, v2, idx, cnt, Bs)
    # rows of blocks 2 and 3 see block 1 as a non-diagonal block
    np.testing.assert_allclose(out1[0, 0, 16:].numpy(), out0[0, 0, 16:].numpy(), rtol=0, atol=1e-6)
    np.testing.assert_allclose(out1[0, 0, :8].numpy(), out0[0, 0, :8].numpy(), rtol=0, atol=0)


def test_block_diagonal_special_case(oracle):
    # ns = 0, nl = 1, k = 0: each block is an independent dense causal problem.
    q, k, v = _qkv(1, 2, 2, 40, 8, 5)
    Bs = 8
    idx, cnt, *_ = oracle.select(q, k, Bs, 0, 1, 0)
    assert idx.shape[-1] == 1 and torch.equal(idx[0, 0, :, 0], torch.arange(5, dtype=torch.int32))
    out, _ = oracle.attn(q, k, v, idx, cnt, Bs)
    for i in range(5):
        sl = slice(i * Bs, (i + 1) * Bs)
        ref = F.scaled_dot_product_attention(q[:, :, sl].float(), k[:, :, sl].float(), v[:, :, sl].float(),
                                             is_causal=True)
        torch.testing.assert_close(out[:, :, sl], ref, rtol=1e-4, atol=2e-5)


def test_single_block_sequence(oracle):
    q, k, v = _qkv(1, 1, 1, 16, 8, 6)
    idx, cnt, *_ = oracle.select(q, k, 16, 1, 4, 8)
    assert idx.shape == (1, 1, 1, 1) and int(cnt) == 1
    out, _ = oracle.attn(q, k, v, idx, cnt, 16)
    ref = F.scaled_dot_product_attention(q.float(), k.float(), v.float(), is_causal=True)
    torch.testing.assert_close(out, ref, rtol=1e-4, atol=2e-5)


def test_row_subset_matches_full(oracle):
    q, k, v = _qkv(2, 4, 2, 32, 8, 7)
    Bs = 4
    idx, cnt, *_ = oracle.select(q, k, Bs, 1, 2, 2)
    full, lse = oracle.attn(q, k, v, idx, cnt, Bs)
    rows = [(1, 3, 7), (0, 0, 0), (1, 2, 4), (0, 3, 5)]
    sub, sl = oracle.attn(q, k, v, idx, cnt, Bs, rows=rows)
    for n, (b, h, i) in enumerate(rows):
        assert torch.equal(sub[n], full[b, h, i * Bs:(i + 1) * Bs])
        assert torch.equal(sl[n], lse[b, h, i * Bs:(i + 1) * Bs])


def test_select_pipeline_invariants_on_workload(oracle):
    """The tiny benchmark workload end to end: selected count = sink + window + k
    clipped to causal, static blocks always present, planted structure irrelevant."""
    from paper_2602_21233_amd import inputs
    w = inputs.workload(0)
    q, k, v = inputs.make_qkv(w)
    idx, cnt, sp, _, _ = oracle.select(q, k, w.block_size, w.n_sink_blocks, w.n_local_blocks, w.top_k_blocks)
    NB = w.n_blocks
    assert idx.shape == (1, 1, NB, w.row_capacity)
    assert cnt[0, 0].tolist() == [min(i + 1, 5) for i in range(NB)]
    assert int(cnt.sum()) == w.visited_pairs == 30
    out, lse = oracle.attn(q, k, v, idx, cnt, w.block_size)
    bf, _ = brute_force(q, k, v, idx, cnt, w.block_size, oracle.default_scale(w.head_dim))
    np.testing.assert_allclose(out.numpy(), bf, rtol=0, atol=1e-6)


# ---- sequence length that is not a multiple of the block size (partial last block) ----

@pytest.mark.parametrize("S,Bs", [(37, 8), (16 * 3 + 1, 16), (5, 8), (63, 16)])
def test_ragged_all_blocks_equals_dense_causal_sdpa(oracle, S, Bs):
    B, Hq, Hkv, D = 1, 4, 2, 16
    q, k, v = _qkv(B, Hq, Hkv, S, D, 60 + S)
    NB = -(-S // Bs)
    idx, cnt = _all_causal(B, Hq, NB)
    out, lse = oracle.attn(q, k, v, idx, cnt, Bs)
    assert out.shape == (B, Hq, S, D) and lse.shape == (B, Hq, S)
    ref = F.scaled_dot_product_attention(q.float(), k.float().repeat_interleave(2, 1), v.float().repeat_interleave(2, 1),
                                         is_causal=True)
    torch.testing.assert_close(out, ref, rtol=1e-4, atol=1e-5)


def test_ragged_equals_the_padded_sequence_on_the_tokens_that_exist(oracle):
    """Causality: tokens appended after the end cannot change the rows before them, so a ragged
    run equals the run on the sequence padded to whole blocks, given the same lists."""
    B, Hq, Hkv, D, Bs, S = 1, 2, 1, 16, 8, 43
    NB = -(-S // Bs)
    qp, kp, vp = _qkv(B, Hq, Hkv, NB * Bs, D, 71)
    q, k, v = qp[:, :, :S].contiguous(), kp[:, :, :S].contiguous(), vp[:, :, :S].contiguous()
    g = torch.Generator().manual_seed(3)
    sp = torch.randn((B, Hq, NB, NB), generator=g)
    idx, cnt = oracle.topk(sp, 1, 2, 2)
    out_r, lse_r = oracle.attn(q, k, v, idx, cnt, Bs)
    out_p, lse_p = oracle.attn(qp, kp, vp, idx, cnt, Bs)
    assert torch.equal(out_r, out_p[:, :, :S]) and torch.equal(lse_r, lse_p[:, :, :S])
    rows = [(0, 1, NB - 1), (0, 0, 2)]
    out_s, lse_s = oracle.attn(q, k, v, idx, cnt, Bs, rows=rows)
    tail = S - (NB - 1) * Bs
    assert torch.equal(out_s[0, :tail], out_r[0, 1, (NB - 1) * Bs:]) and (out_s[0, tail:] == 0).all()
    assert torch.equal(out_s[1], out_r[0, 0, 2 * Bs:3 * Bs])


def test_ragged_pooling_averages_the_tokens_that_exist(oracle):
    Bs, D, S = 8, 16, 29
    x = torch.randn((2, 3, S, D), generator=torch.Generator().manual_seed(4)).to(torch.bfloat16)
    got = oracle.pool(x, Bs)
    assert got.shape == (2, 3, 4, D)
    xd = x.double().numpy()
    for i in range(4):
        want = xd[:, :, i * Bs:min((i + 1) * Bs, S)].mean(axis=2)
        np.testing.assert_allclose(got[:, :, i].numpy(), want, rtol=1e-6, atol=1e-7)
    vn = oracle.vnorm(x, Bs)
    want = np.linalg.norm(xd[:, :, 24:29], axis=-1).mean(-1)
    np.testing.assert_allclose(vn[:, :, 3].numpy(), want, rtol=2e-7)


# ---- KV prefix (chunked prefill): the queries are the last tokens of a longer sequence ----

@pytest.mark.parametrize("Sq,P,Bs", [(24, 16, 8), (19, 32, 8), (8, 8, 8), (33, 48, 16)])
def test_prefix_call_equals_the_rows_of_the_full_run(oracle, Sq, P, Bs):
    """Every step is local to a query block, so running only the last Sq tokens against the full
    K/V must reproduce the full run's rows: pooled scores, lists and attention."""
    B, Hq, Hkv, D, ns, nl, k = 1, 4, 2, 16, 1, 2, 2
    S = P + Sq
    q, kk, v = _qkv(B, Hq, Hkv, S, D, 80 + Sq)
    off = P // Bs
    idx_f, cnt_f, sp_f, *_ = oracle.select(q, kk, Bs, ns, nl, k, v=v)
    out_f, lse_f = oracle.attn(q, kk, v, idx_f, cnt_f, Bs)
    qc = q[:, :, P:].contiguous()
    idx_c, cnt_c, sp_c, *_ = oracle.select(qc, kk, Bs, ns, nl, k, v=v)
    assert sp_c.shape == (B, Hq, -(-Sq // Bs), -(-S // Bs))
    assert torch.equal(sp_c, sp_f[:, :, off:]) and torch.equal(idx_c, idx_f[:, :, off:]) and torch.equal(cnt_c, cnt_f[:, :, off:])
    out_c, lse_c = oracle.attn(qc, kk, v, idx_c, cnt_c, Bs)
    assert torch.equal(out_c, out_f[:, :, P:]) and torch.equal(lse_c, lse_f[:, :, P:])


def test_prefix_all_blocks_equals_dense_causal_rows(oracle):
    B, Hq, Hkv, D, Bs, P, Sq = 1, 2, 1, 16, 8, 24, 21
    S = P + Sq
    q, kk, v = _qkv(B, Hq, Hkv, S, D, 91)
    qc = q[:, :, P:].contiguous()
    NBq, NBk = -(-Sq // Bs), -(-S // Bs)
    sp = torch.zeros((B, Hq, NBq, NBk))
    idx, cnt = oracle.topk(sp, 0, 1, NBk)
    assert all(int(cnt[0, 0, i]) == i + P // Bs + 1 for i in range(NBq))
    out, _ = oracle.attn(qc, kk, v, idx, cnt, Bs)
    ref = F.scaled_dot_product_attention(q.float(), kk.float().repeat_interleave(2, 1), v.float().repeat_interleave(2, 1),
                                         is_causal=True)[:, :, P:]
    torch.testing.assert_close(out, ref, rtol=1e-4, atol=1e-5)
