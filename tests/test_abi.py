"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every symbol the header declares, and rejects bad arguments before any launch."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2602_21233_amd as m
    return m.load_library()


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "sparse_prefill.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(spa_[a-z_]+|sparse_prefill_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_symbols()
    assert {"sparse_prefill_select", "sparse_prefill_attn", "sparse_prefill_fused",
            "sparse_prefill_topk_from_scores", "sparse_prefill_pool", "spa_workspace_bytes",
            "spa_row_capacity", "spa_strerror"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    from paper_2602_21233_amd import binding
    assert sorted(binding.EXPORTS) == names


def _params(**kw):
    from paper_2602_21233_amd import binding
    base = dict(batch=1, n_q_heads=4, n_kv_heads=2, seq_len=1024, head_dim=128, block_size=128,
                n_sink_blocks=1, n_local_blocks=2, top_k_blocks=3)
    base.update(kw)
    p = binding.make_params(**base)
    for f in ("q_stride", "k_stride", "v_stride", "o_stride"):
        setattr(p, f, (ctypes.c_int64 * 3)(0, base["seq_len"] * base["head_dim"], base["head_dim"]))
    return p


def test_row_capacity_and_workspace(lib):
    import paper_2602_21233_amd as m
    assert m.row_capacity(_params()) == 6
    assert m.row_capacity(_params(top_k_blocks=100)) == 8          # clipped to NB
    assert m.row_capacity(_params(top_k_blocks=0)) == 3
    assert m.row_capacity(_params(stride_blocks=3)) == 8           # 6 + (8 - 1) // 3
    assert m.row_capacity(_params(top_k_blocks=0, stride_blocks=4)) == 4
    assert m.row_capacity(_params(n_dense_q_blocks=2)) == 8        # a dense strip needs full rows
    assert m.row_capacity(_params(seq_len=1000, top_k_blocks=100)) == 8   # 7 whole blocks + a partial one
    assert m.row_capacity(_params(seq_len=1025, top_k_blocks=100)) == 9
    assert m.row_capacity(_params(kv_prefix_len=512, top_k_blocks=100)) == 12     # 4 prefix + 8 query blocks
    assert m.row_capacity(_params(top_k_blocks=0, stride_blocks=2, stride_reach_blocks=5)) == 5   # 3 + (5 - 1) // 2
    ws = m.workspace_bytes(_params())
    # pooled Q (4*8*128 fp32) + pooled K (2*8*128 fp32) + lists + transposed V (2*1024*128 bf16),
    # each 256-byte aligned
    assert ws >= 4 * 8 * 128 * 4 + 2 * 8 * 128 * 4 + 4 * 8 * 6 * 4 + 4 * 8 * 4 + 2 * 1024 * 128 * 2 and ws % 256 == 0


@pytest.mark.parametrize("kw,code", [
    (dict(head_dim=96), -2), (dict(block_size=32), -2), (dict(seq_len=0), -2),
    (dict(n_q_heads=5), -2), (dict(batch=0), -2), (dict(seq_len=128 * 4097), -2),
    (dict(n_local_blocks=0), -3), (dict(n_sink_blocks=-1), -3), (dict(top_k_blocks=-2), -3),
    (dict(stride_blocks=-1), -3), (dict(n_dense_q_blocks=-4), -3), (dict(stride_reach_blocks=-1), -3), (dict(lists_per_kv_head=2), -3),
    (dict(kv_prefix_len=-128), -2), (dict(kv_prefix_len=100), -2), (dict(kv_prefix_len=128 * 4090), -2),
    (dict(softmax_scale=-1.0), -2),
])
def test_bad_params_rejected_on_host(lib, kw, code):
    p = _params(**kw)
    t = ctypes.c_int32()
    assert lib.spa_row_capacity(ctypes.byref(p), ctypes.byref(t)) == code
    n = ctypes.c_size_t()
    assert lib.spa_workspace_bytes(ctypes.byref(p), ctypes.byref(n)) == code
    assert lib.spa_strerror(code).decode() not in ("ok", "unknown error code")


def test_null_and_misaligned_pointers_rejected_before_launch(lib):
    p = _params()
    fake = ctypes.c_void_p(0x10000)            # never dereferenced on the host
    assert lib.sparse_prefill_attn(ctypes.byref(p), None, fake, fake, fake, fake, fake, None, fake, 1 << 30, None) == -1
    assert lib.sparse_prefill_attn(ctypes.byref(p), fake, fake, fake, None, fake, fake, None, fake, 1 << 30, None) == -1
    assert lib.sparse_prefill_attn(ctypes.byref(p), ctypes.c_void_p(0x10008), fake, fake, fake, fake, fake,
                                   None, fake, 1 << 30, None) == -4
    assert lib.sparse_prefill_attn(ctypes.byref(p), fake, fake, fake, fake, fake, fake, None, fake, 64, None) == -5
    assert lib.sparse_prefill_select(ctypes.byref(p), fake, fake, fake, fake, None, None, 1 << 30, None) == -1
    assert lib.sparse_prefill_select(ctypes.byref(p), fake, fake, fake, fake, None, fake, 16, None) == -5
    assert lib.sparse_prefill_fused(ctypes.byref(p), fake, fake, fake, fake, None, fake, None, fake, 1 << 30,
                                    None) == -1
    assert lib.sparse_prefill_topk_from_scores(ctypes.byref(p), None, fake, fake, None) == -1
    assert lib.sparse_prefill_pool(ctypes.byref(p), fake, None, None, None, None) == -1
    # the budget-schedule calls: a missing schedule is an error, the other checks are those of the uniform calls
    assert lib.sparse_prefill_select_tpd(ctypes.byref(p), fake, fake, None, fake, fake, None, fake, 1 << 30, None) == -1
    assert lib.sparse_prefill_select_tpd(ctypes.byref(p), fake, fake, fake, fake, fake, None, fake, 16, None) == -5
    assert lib.sparse_prefill_topk_from_scores_tpd(ctypes.byref(p), fake, None, fake, fake, None) == -1
    assert lib.sparse_prefill_topk_from_scores_tpd(ctypes.byref(p), None, fake, fake, fake, None) == -1
    assert lib.sparse_prefill_fused_tpd(ctypes.byref(p), fake, fake, fake, None, fake, None, None, None, fake,
                                        1 << 30, None) == -1
    assert lib.sparse_prefill_fused_tpd(ctypes.byref(p), fake, fake, fake, fake, fake, None, fake, None, fake,
                                        1 << 30, None) == -1
    # output-aware calls: V is required
    assert lib.sparse_prefill_select_stem(ctypes.byref(p), fake, fake, None, None, fake, fake, None, fake, 1 << 30,
                                          None) == -1
    assert lib.sparse_prefill_select_stem(ctypes.byref(p), fake, fake, ctypes.c_void_p(0x10008), None, fake, fake,
                                          None, fake, 1 << 30, None) == -4
    assert lib.sparse_prefill_fused_stem(ctypes.byref(p), fake, fake, None, None, fake, None, None, None, fake,
                                         1 << 30, None) == -1
    assert lib.sparse_prefill_value_norms(ctypes.byref(p), fake, None, None) == -1
    assert lib.sparse_prefill_value_norms(ctypes.byref(p), None, fake, None) == -1
    # general form: a NULL opts is the plain call, argument checks are unchanged
    from paper_2602_21233_amd import binding
    o = binding.SpaSelectOpts()
    assert lib.sparse_prefill_select_ex(ctypes.byref(p), fake, fake, None, fake, fake, None, None, 1 << 30, None) == -1
    assert lib.sparse_prefill_select_ex(ctypes.byref(p), fake, fake, ctypes.byref(o), fake, fake, None, fake, 16,
                                        None) == -5
    o.v = 0x10008
    assert lib.sparse_prefill_select_ex(ctypes.byref(p), fake, fake, ctypes.byref(o), fake, fake, None, fake,
                                        1 << 30, None) == -4
    assert lib.sparse_prefill_topk_from_scores_ex(ctypes.byref(p), None, None, fake, fake, None) == -1
    # cumulative-mass budget: negative or NaN is an error, found before any launch
    for bad_gamma in (-0.5, float("nan")):
        o2 = binding.SpaSelectOpts()
        o2.mass_gamma = bad_gamma
        assert lib.sparse_prefill_select_ex(ctypes.byref(p), fake, fake, ctypes.byref(o2), fake, fake, None, fake,
                                            1 << 30, None) == -3
        assert lib.sparse_prefill_topk_from_scores_ex(ctypes.byref(p), fake, ctypes.byref(o2), fake, fake, None) == -3
        assert lib.sparse_prefill_fused_ex(ctypes.byref(p), fake, fake, fake, ctypes.byref(o2), fake, None, fake, fake,
                                           fake, 1 << 30, None) == -3
    assert lib.sparse_prefill_fused_ex(ctypes.byref(p), fake, fake, fake, None, fake, None, fake, None, fake,
                                       1 << 30, None) == -1
    bad = _params()
    bad.q_stride = (ctypes.c_int64 * 3)(0, 1024 * 128, 100)
    assert lib.sparse_prefill_attn(ctypes.byref(bad), fake, fake, fake, fake, fake, fake, None, fake, 1 << 30, None) == -4
    assert lib.spa_strerror(0).decode() == "ok"
    assert lib.spa_strerror(-99).decode() == "unknown error code"


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_check_lists_rejects_null_pointers_and_bad_shapes(lib):
    p = _params()
    fake = ctypes.c_void_p(256)
    assert lib.sparse_prefill_check_lists(ctypes.byref(p), None, fake, fake, None) == -1
    assert lib.sparse_prefill_check_lists(ctypes.byref(p), fake, None, fake, None) == -1
    assert lib.sparse_prefill_check_lists(ctypes.byref(p), fake, fake, None, None) == -1
    assert lib.sparse_prefill_check_lists(ctypes.byref(_params(head_dim=96)), fake, fake, fake, None) == -2
