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


def test_static_scratch_select_rejects_what_does_not_fit(lib):
    """The size check of the call that allocates nothing is made on the host, before the array's address
    is even asked for: nothing is enqueued and no GPU is needed."""
    from paper_2602_21233_amd import binding
    fake = ctypes.c_void_p(0x10000)                       # never dereferenced: the size check comes first
    # 16 KV heads x 2048 key blocks x head_dim 128 x 4 bytes = 16 MiB of pooled K: twice the array
    p = binding.make_params(batch=1, n_q_heads=16, n_kv_heads=16, seq_len=2048 * 128, head_dim=128, block_size=128,
                            n_sink_blocks=1, n_local_blocks=2, top_k_blocks=8)
    for f in ("q_stride", "k_stride"):
        setattr(p, f, (ctypes.c_int64 * 3)(0, 2048 * 128 * 128, 128))
    assert lib.sparse_prefill_select_static(ctypes.byref(p), fake, fake, fake, fake, None, None) == -7
    assert b"static" in lib.spa_strerror(-7)
    # exactly at the limit (8 KV heads) the size check passes and the next check (here: a NULL output) answers
    p.n_q_heads, p.n_kv_heads = 8, 8
    assert lib.sparse_prefill_select_static(ctypes.byref(p), fake, fake, None, fake, None, None) == -1
    # group-shared lists add the pooled queries: 32 + 8 heads x 1024 blocks x 128 x 4 = 20 MiB
    p = binding.make_params(batch=1, n_q_heads=32, n_kv_heads=8, seq_len=1024 * 128, head_dim=128, block_size=128,
                            n_sink_blocks=1, n_local_blocks=4, top_k_blocks=64, lists_per_kv_head=1)
    for f in ("q_stride", "k_stride"):
        setattr(p, f, (ctypes.c_int64 * 3)(0, 1024 * 128 * 128, 128))
    assert lib.sparse_prefill_select_static(ctypes.byref(p), fake, fake, fake, fake, None, None) == -7


def test_kept_vt_calls_reject_bad_arguments_on_the_host(lib):
    p = _params()                                          # 8 key blocks of 128 tokens
    fake = ctypes.c_void_p(0x10000)
    i64, i32 = ctypes.c_int64, ctypes.c_int32
    assert lib.sparse_prefill_transpose_v(ctypes.byref(p), fake, None, i64(8), i32(0), i32(8), None) == -1
    assert lib.sparse_prefill_transpose_v(ctypes.byref(p), None, fake, i64(8), i32(0), i32(8), None) == -1
    assert lib.sparse_prefill_transpose_v(ctypes.byref(p), fake, ctypes.c_void_p(0x10008), i64(8), i32(0), i32(8), None) == -4
    assert lib.sparse_prefill_transpose_v(ctypes.byref(p), fake, fake, i64(7), i32(0), i32(7), None) == -2      # allocation too short
    assert lib.sparse_prefill_transpose_v(ctypes.byref(p), fake, fake, i64(8), i32(3), i32(6), None) == -2      # past the last block
    assert lib.sparse_prefill_transpose_v(ctypes.byref(p), fake, fake, i64(8), i32(-1), i32(2), None) == -2
    assert lib.sparse_prefill_transpose_v(ctypes.byref(p), fake, fake, i64(8), i32(2), i32(-1), None) == -2
    assert lib.sparse_prefill_transpose_v(ctypes.byref(_params(head_dim=96)), fake, fake, i64(8), i32(0), i32(8), None) == -2
    assert lib.sparse_prefill_attn_vt(ctypes.byref(p), fake, fake, None, i64(8), fake, fake, fake, None, None) == -1
    assert lib.sparse_prefill_attn_vt(ctypes.byref(p), fake, fake, fake, i64(8), None, fake, fake, None, None) == -1
    assert lib.sparse_prefill_attn_vt(ctypes.byref(p), fake, fake, fake, i64(7), fake, fake, fake, None, None) == -2
    assert lib.sparse_prefill_attn_vt(ctypes.byref(p), fake, fake, ctypes.c_void_p(0x10004), i64(8), fake, fake, fake, None, None) == -4
    assert lib.sparse_prefill_attn_vt(ctypes.byref(p), None, fake, fake, i64(8), fake, fake, fake, None, None) == -1


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


def _compile_and_run_c(tmp_path, body, std="-std=c99"):
    import subprocess
    src = tmp_path / "t.c"
    src.write_text(body)
    exe = tmp_path / "t"
    subprocess.run(["gcc", std, "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe), "-ldl"], check=True, capture_output=True, text=True)
    return subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout


def test_header_is_plain_c_and_the_binding_mirrors_its_structs(tmp_path):
    """The header compiles as strict C99 with no other include, and the ctypes structures have
    the size and the field offsets a C compiler gives the header's structs."""
    from paper_2602_21233_amd import binding
    lines = ['#include "sparse_prefill.h"', "#include <stdio.h>", "int main(void) {",
             '  printf("spa_params %zu\\n", sizeof(spa_params));',
             '  printf("spa_select_opts %zu\\n", sizeof(spa_select_opts));']
    for struct, cls in (("spa_params", binding.SpaParams), ("spa_select_opts", binding.SpaSelectOpts)):
        for name, _ in cls._fields_:
            lines.append(f'  printf("{struct}.{name} %zu\\n", offsetof({struct}, {name}));')
    lines += ["  return SPA_OK;", "}"]
    got = dict(l.split() for l in _compile_and_run_c(tmp_path, "\n".join(lines)).splitlines())
    assert int(got["spa_params"]) == ctypes.sizeof(binding.SpaParams)
    assert int(got["spa_select_opts"]) == ctypes.sizeof(binding.SpaSelectOpts)
    for struct, cls in (("spa_params", binding.SpaParams), ("spa_select_opts", binding.SpaSelectOpts)):
        for name, _ in cls._fields_:
            assert int(got[f"{struct}.{name}"]) == getattr(cls, name).offset, (struct, name)


def test_library_is_callable_from_plain_c(tmp_path, lib):
    """A C program with no Python and no torch loads the library and gets the host-side answers."""
    from paper_2602_21233_amd import binding
    body = r'''
#define _POSIX_C_SOURCE 200809L
#include "sparse_prefill.h"
#include <dlfcn.h>
#include <stdio.h>
#include <string.h>
typedef int (*cap_fn)(const spa_params *, int32_t *);
typedef int (*ws_fn)(const spa_params *, size_t *);
typedef const char *(*err_fn)(int);
typedef int (*attn_fn)(const spa_params *, const void *, const void *, const void *, const int32_t *, const int32_t *,
                       void *, float *, void *, size_t, void *);
int main(void) {
    void *h = dlopen("%LIB%", RTLD_NOW);
    if (!h) { printf("dlopen failed: %s\n", dlerror()); return 1; }
    cap_fn cap; ws_fn ws; err_fn err; attn_fn attn;
    *(void **)&cap = dlsym(h, "spa_row_capacity");
    *(void **)&ws = dlsym(h, "spa_workspace_bytes");
    *(void **)&err = dlsym(h, "spa_strerror");
    *(void **)&attn = dlsym(h, "sparse_prefill_attn");
    if (!cap || !ws || !err || !attn) { printf("missing symbol\n"); return 1; }
    spa_params p;
    memset(&p, 0, sizeof p);
    p.batch = 1; p.n_q_heads = 32; p.n_kv_heads = 8; p.seq_len = 131072; p.head_dim = 128; p.block_size = 128;
    p.n_sink_blocks = 1; p.n_local_blocks = 4; p.top_k_blocks = 64;
    int32_t T = -1; size_t bytes = 0;
    int rc1 = cap(&p, &T), rc2 = ws(&p, &bytes);
    printf("cap %d %d\nws %d %zu\n", rc1, (int)T, rc2, bytes);
    printf("attn_null %d\n", attn(&p, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, 0, NULL));
    p.head_dim = 96;
    printf("bad_shape %d %s\n", cap(&p, &T), err(cap(&p, &T)));
    return 0;
}
'''.replace("%LIB%", binding.library_path())
    out = _compile_and_run_c(tmp_path, body, std="-std=c99").splitlines()
    assert out[0] == "cap 0 69"
    rc, nbytes = out[1].split()[1:]
    p = _params(n_q_heads=32, n_kv_heads=8, seq_len=131072, n_local_blocks=4, top_k_blocks=64)
    import paper_2602_21233_amd as m
    assert int(rc) == 0 and int(nbytes) == m.workspace_bytes(p)
    assert out[2] == "attn_null -1"
    assert out[3].startswith("bad_shape -2 ") and len(out[3]) > len("bad_shape -2 ")
