"""Pins for the oracle's ragged-batch wrappers (a batch whose entries have different lengths: each
entry is, by definition, a batch-1 problem of its own length; Sec. 4.1 describes prefill of one
sequence, batching is a deployment matter the paper leaves open).  The wrappers only slice and
call the pinned single-sequence functions; pinned here: equal lengths reproduce the plain batch
call bit for bit, an entry's result depends on nothing outside its own tokens, and the padded rows
come back empty."""
import torch


def _qkv(B, Hq, Hkv, S, Skv, D, seed):
    g = torch.Generator().manual_seed(seed)
    q = torch.randn((B, Hq, S, D), generator=g).to(torch.bfloat16)
    k = torch.randn((B, Hkv, Skv, D), generator=g).to(torch.bfloat16)
    v = torch.randn((B, Hkv, Skv, D), generator=g).to(torch.bfloat16)
    return q, k, v


def test_equal_lengths_reproduce_the_batch_call(oracle):
    B, Hq, Hkv, S, D, Bs = 2, 4, 2, 5 * 32 + 9, 32, 32
    q, k, v = _qkv(B, Hq, Hkv, S, S, D, 1)
    idx, cnt, *_ = oracle.select(q, k, Bs, 1, 2, 2)
    r_idx, r_cnt = oracle.select_ragged(q, k, [S, S], Bs, 1, 2, 2)
    assert torch.equal(idx, r_idx) and torch.equal(cnt, r_cnt)
    out, lse = oracle.attn(q, k, v, idx, cnt, Bs)
    r_out, r_lse = oracle.attn_ragged(q, k, v, r_idx, r_cnt, [S, S], Bs)
    assert torch.equal(out, r_out) and torch.equal(lse, r_lse)


def test_an_entry_depends_only_on_its_own_tokens(oracle):
    B, Hq, Hkv, S, P, D, Bs = 3, 2, 1, 4 * 32, 2 * 32, 32, 32
    lens = [S, 70, 33]
    q, k, v = _qkv(B, Hq, Hkv, S, P + S, D, 2)
    idx, cnt = oracle.select_ragged(q, k, lens, Bs, 1, 2, 1, v=v)
    out, lse = oracle.attn_ragged(q, k, v, idx, cnt, lens, Bs)
    q2, k2, v2 = q.clone(), k.clone(), v.clone()
    for b, n in enumerate(lens):                     # scribble over the padding and over entry 0
        q2[b, :, n:] = 7.0
        k2[b, :, P + n:] = -3.0
        v2[b, :, P + n:] = 100.0
    q2[0], k2[0], v2[0] = q[0].flip(1), k[0].flip(1), v[0].flip(1)
    idx2, cnt2 = oracle.select_ragged(q2, k2, lens, Bs, 1, 2, 1, v=v2)
    out2, lse2 = oracle.attn_ragged(q2, k2, v2, idx2, cnt2, lens, Bs)
    for b in (1, 2):
        n = lens[b]
        assert torch.equal(idx[b], idx2[b]) and torch.equal(cnt[b], cnt2[b])
        assert torch.equal(out[b, :, :n], out2[b, :, :n]) and torch.equal(lse[b, :, :n], lse2[b, :, :n])
    # padded rows: empty lists, no output
    for b, n in enumerate(lens):
        nb = -(-n // Bs)
        assert (cnt[b, :, nb:] == 0).all() and (idx[b, :, nb:] == -1).all()
        assert (cnt[b, :, :nb] > 0).all()
        assert torch.isnan(out[b, :, n:]).all() and not torch.isnan(out[b, :, :n]).any()
    # an entry equals the single-sequence call on its slice (the definition, spelled out once)
    n = lens[1]
    i1, c1, *_ = oracle.select(q[1:2, :, :n], k[1:2, :, :P + n], Bs, 1, 2, 1, v=v[1:2, :, :P + n])
    assert torch.equal(idx[1, :, :i1.shape[2], :i1.shape[3]], i1[0]) and torch.equal(cnt[1, :, :c1.shape[2]], c1[0])
