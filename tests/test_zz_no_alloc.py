"""The select call that allocates nothing (sparse_prefill_select_static, for callers that cannot
call hipMalloc or hand over a workspace) against the workspace call it is a variant of: same lists
and same scores, bit for bit, on two calls in a row of which the second is smaller, so that the
static scratch still holds the first call's pooled keys when the second one runs."""
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def spa():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2602_21233_amd as m
    m.load_library()
    return m


def _qk(B, Hq, Hkv, S, Skv, D, seed):
    g = torch.Generator().manual_seed(seed)
    q = torch.randn((B, Hq, S, D), generator=g).to(torch.bfloat16)
    k = torch.randn((B, Hkv, Skv, D), generator=g).to(torch.bfloat16)
    return q.cuda(), k.cuda()


def test_static_scratch_select_equals_the_workspace_call_twice_in_a_row(spa, oracle):
    # first call: 40 blocks of 128 tokens, 8/2 heads; second call: smaller in every respect
    # (fewer heads, 17 blocks of 64 tokens + a partial one, head_dim 64, a KV prefix)
    calls = [dict(B=2, Hq=8, Hkv=2, S=40 * 128, P=0, D=128, Bs=128, ns=1, nl=2, k=9, seed=501),
             dict(B=1, Hq=2, Hkv=1, S=17 * 64 + 30, P=3 * 64, D=64, Bs=64, ns=2, nl=3, k=5, seed=502)]
    for c in calls:
        q, k = _qk(c["B"], c["Hq"], c["Hkv"], c["S"], c["P"] + c["S"], c["D"], c["seed"])
        want_idx, want_cnt, want_sp = spa.select(q, k, c["Bs"], c["ns"], c["nl"], c["k"], return_scores=True)
        # the caller's own output buffers: the static call itself must not need an allocation
        idx = torch.full_like(want_idx, -7)
        cnt = torch.full_like(want_cnt, -7)
        torch.cuda.synchronize()
        before = torch.cuda.memory_stats()["allocation.all.allocated"]
        got_idx, got_cnt = spa.select_static(q, k, c["Bs"], c["ns"], c["nl"], c["k"], block_idx=idx, block_cnt=cnt)
        assert torch.cuda.memory_stats()["allocation.all.allocated"] == before      # no torch allocation either
        torch.cuda.synchronize()
        assert torch.equal(got_cnt, want_cnt) and torch.equal(got_idx, want_idx), c
        _, _, got_sp = spa.select_static(q, k, c["Bs"], c["ns"], c["nl"], c["k"], return_scores=True)
        assert torch.equal(got_sp, want_sp), c                                     # -inf == -inf; no NaN here
        # and, like the workspace call, exactly the rule applied to its own scores
        o_idx, o_cnt = oracle.topk(got_sp.cpu(), c["ns"], c["nl"], c["k"])
        assert torch.equal(got_idx.cpu(), o_idx) and torch.equal(got_cnt.cpu(), o_cnt), c


def test_static_scratch_select_group_shared_and_ragged(spa):
    q, k = _qk(2, 4, 2, 21 * 64, 21 * 64, 128, 503)
    lens = torch.tensor([21 * 64, 9 * 64 + 5], dtype=torch.int32).cuda()
    for kw in (dict(group_shared=True), dict(seq_lens=lens), dict(group_shared=True, seq_lens=lens)):
        want_idx, want_cnt = spa.select(q, k, 64, 1, 4, 6, **kw)
        got_idx, got_cnt = spa.select_static(q, k, 64, 1, 4, 6, **kw)
        assert torch.equal(got_cnt, want_cnt) and torch.equal(got_idx, want_idx), kw


def test_static_scratch_select_replays_from_a_hip_graph(spa):
    """What the call is for: recorded into a HIP graph (its first call on the device, which looks the
    array's address up, was made before the capture), then replayed with eager work and
    synchronisations in between; every replay reproduces the eager lists."""
    q, k = _qk(1, 4, 2, 40 * 128, 40 * 128, 128, 504)
    Bs, ns, nl, tk = 128, 1, 2, 6
    want_idx, want_cnt = spa.select(q, k, Bs, ns, nl, tk)
    idx, cnt = torch.empty_like(want_idx), torch.empty_like(want_cnt)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        spa.select_static(q, k, Bs, ns, nl, tk, block_idx=idx, block_cnt=cnt)       # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=s):
        spa.select_static(q, k, Bs, ns, nl, tk, block_idx=idx, block_cnt=cnt)
    for rep in range(3):
        idx.fill_(-5)
        cnt.fill_(-5)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(idx, want_idx) and torch.equal(cnt, want_cnt), rep
        q2, k2 = _qk(1, 2, 1, 9 * 64, 9 * 64, 64, 505 + rep)                    # eager work on the same array in between
        spa.select_static(q2, k2, 64, 1, 1, 2)
        torch.cuda.synchronize()
