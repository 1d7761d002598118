"""ctypes binding of include/sparse_prefill.h.  Same names, argument marshalling
only.  There is no fallback: without the built HIP library every call raises."""
from __future__ import annotations

import ctypes
import os

import torch  # imported before the library so both share one HIP runtime

from . import build as _build

_lib = None

EXPORTS = ("spa_strerror", "spa_row_capacity", "spa_workspace_bytes", "sparse_prefill_pool",
           "sparse_prefill_select", "sparse_prefill_topk_from_scores", "sparse_prefill_attn",
           "sparse_prefill_fused", "sparse_prefill_select_tpd", "sparse_prefill_topk_from_scores_tpd",
           "sparse_prefill_fused_tpd", "sparse_prefill_value_norms", "sparse_prefill_select_stem",
           "sparse_prefill_fused_stem", "sparse_prefill_select_ex", "sparse_prefill_topk_from_scores_ex",
           "sparse_prefill_fused_ex", "sparse_prefill_check_lists", "sparse_prefill_select_static",
           "sparse_prefill_transpose_v", "sparse_prefill_attn_vt")


class SpaError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"sparse_prefill error {code}: {text}")
        self.code = code


class SpaParams(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("seq_len", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("block_size", ctypes.c_int32),
                ("n_sink_blocks", ctypes.c_int32), ("n_local_blocks", ctypes.c_int32),
                ("top_k_blocks", ctypes.c_int32), ("softmax_scale", ctypes.c_float),
                ("q_stride", ctypes.c_int64 * 3), ("k_stride", ctypes.c_int64 * 3),
                ("v_stride", ctypes.c_int64 * 3), ("o_stride", ctypes.c_int64 * 3),
                ("stride_blocks", ctypes.c_int32), ("n_dense_q_blocks", ctypes.c_int32),
                ("stride_reach_blocks", ctypes.c_int32), ("kv_prefix_len", ctypes.c_int32),
                ("lists_per_kv_head", ctypes.c_int32), ("seq_lens", ctypes.c_void_p)]


class SpaSelectOpts(ctypes.Structure):
    _fields_ = [("top_k_per_block", ctypes.c_void_p), ("v", ctypes.c_void_p), ("head_pattern", ctypes.c_void_p),
                ("mass_gamma", ctypes.c_float)]


def library_path() -> str:
    return _build.LIB


def load_library():
    """Load the built library; build it first only if nothing is built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB):
        _build.build_library()
    lib = ctypes.CDLL(_build.LIB)
    vp, pp = ctypes.c_void_p, ctypes.POINTER(SpaParams)
    lib.spa_strerror.restype = ctypes.c_char_p
    lib.spa_strerror.argtypes = [ctypes.c_int]
    lib.spa_row_capacity.argtypes = [pp, ctypes.POINTER(ctypes.c_int32)]
    lib.spa_workspace_bytes.argtypes = [pp, ctypes.POINTER(ctypes.c_size_t)]
    lib.sparse_prefill_pool.argtypes = [pp, vp, vp, vp, vp, vp]
    lib.sparse_prefill_select.argtypes = [pp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.sparse_prefill_select_static.argtypes = [pp, vp, vp, vp, vp, vp, vp]
    lib.sparse_prefill_topk_from_scores.argtypes = [pp, vp, vp, vp, vp]
    lib.sparse_prefill_attn.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.sparse_prefill_check_lists.argtypes = [pp, vp, vp, vp, vp]
    lib.sparse_prefill_transpose_v.argtypes = [pp, vp, vp, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, vp]
    lib.sparse_prefill_attn_vt.argtypes = [pp, vp, vp, vp, ctypes.c_int64, vp, vp, vp, vp, vp]
    lib.sparse_prefill_fused.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.sparse_prefill_select_tpd.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.sparse_prefill_topk_from_scores_tpd.argtypes = [pp, vp, vp, vp, vp, vp]
    lib.sparse_prefill_fused_tpd.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.sparse_prefill_value_norms.argtypes = [pp, vp, vp, vp]
    lib.sparse_prefill_select_stem.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.sparse_prefill_fused_stem.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    po = ctypes.POINTER(SpaSelectOpts)
    lib.sparse_prefill_select_ex.argtypes = [pp, vp, vp, po, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.sparse_prefill_topk_from_scores_ex.argtypes = [pp, vp, po, vp, vp, vp]
    lib.sparse_prefill_fused_ex.argtypes = [pp, vp, vp, vp, po, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    for name in EXPORTS[1:]:
        getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def _check(rc: int):
    if rc != 0:
        raise SpaError(rc, load_library().spa_strerror(rc).decode())


def _strides(t):
    if t is None:
        return (ctypes.c_int64 * 3)(0, 0, 0)
    assert t.dim() == 4 and t.stride(3) == 1, "head_dim axis must be contiguous"
    return (ctypes.c_int64 * 3)(t.stride(0), t.stride(1), t.stride(2))


def make_params(*, batch, n_q_heads, n_kv_heads, seq_len, head_dim, block_size, n_sink_blocks,
                n_local_blocks, top_k_blocks, softmax_scale=None, q=None, k=None, v=None, out=None,
                stride_blocks=0, n_dense_q_blocks=0, stride_reach_blocks=0, lists_per_kv_head=0, kv_prefix_len=0,
                seq_lens=None) -> SpaParams:
    """seq_lens: optional int32 device tensor [batch] (ragged batch); the caller keeps it alive."""
    p = SpaParams()
    if seq_lens is not None:
        if seq_lens.dtype != torch.int32 or not seq_lens.is_cuda or not seq_lens.is_contiguous() \
                or tuple(seq_lens.shape) != (batch,):
            raise TypeError("seq_lens must be a contiguous int32 device tensor of shape [batch]")
        p.seq_lens = seq_lens.data_ptr()
    p.batch, p.n_q_heads, p.n_kv_heads = batch, n_q_heads, n_kv_heads
    p.seq_len, p.head_dim, p.block_size = seq_len, head_dim, block_size
    p.n_sink_blocks, p.n_local_blocks, p.top_k_blocks = n_sink_blocks, n_local_blocks, top_k_blocks
    p.stride_blocks, p.n_dense_q_blocks = stride_blocks, n_dense_q_blocks
    p.stride_reach_blocks = stride_reach_blocks
    p.lists_per_kv_head = int(lists_per_kv_head)
    p.kv_prefix_len = kv_prefix_len
    p.softmax_scale = 0.0 if softmax_scale is None else float(softmax_scale)
    p.q_stride, p.k_stride, p.v_stride, p.o_stride = _strides(q), _strides(k), _strides(v), _strides(out)
    return p


def _params_from(q, k, block_size, ns, nl, topk, scale, v=None, out=None, stride_blocks=0,
                 n_dense_q_blocks=0, stride_reach_blocks=0, group_shared=False, seq_lens=None) -> SpaParams:
    B, Hq, S, D = q.shape
    return make_params(batch=B, n_q_heads=Hq, n_kv_heads=k.shape[1], seq_len=S, head_dim=D,
                       block_size=block_size, n_sink_blocks=ns, n_local_blocks=nl, top_k_blocks=topk,
                       softmax_scale=scale, q=q, k=k, v=v, out=out, stride_blocks=stride_blocks,
                       n_dense_q_blocks=n_dense_q_blocks, stride_reach_blocks=stride_reach_blocks,
                       lists_per_kv_head=group_shared, kv_prefix_len=k.shape[2] - S, seq_lens=seq_lens)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(ref):
    return ctypes.c_void_p(torch.cuda.current_stream(ref.device).cuda_stream)


def _dev_bf16(*ts):
    for t in ts:
        if t.dtype != torch.bfloat16 or not t.is_cuda:
            raise TypeError("expected bf16 tensors on the GPU")


def _schedule(top_k_per_block, n_blocks, device):
    t = top_k_per_block
    if t.dtype != torch.int32 or not t.is_cuda or not t.is_contiguous() or tuple(t.shape) != (n_blocks,):
        raise TypeError("top_k_per_block must be a contiguous int32 tensor [NB] on the GPU")
    return t


def _head_pattern(hp, n_q_heads):
    if hp.dtype != torch.int32 or not hp.is_cuda or not hp.is_contiguous() or tuple(hp.shape) != (n_q_heads, 3):
        raise TypeError("head_pattern must be a contiguous int32 tensor [n_q_heads, 3] on the GPU")
    return hp


def _opts(top_k_per_block=None, v=None, head_pattern=None, mass_gamma=None) -> SpaSelectOpts:
    o = SpaSelectOpts()
    o.mass_gamma = 0.0 if mass_gamma is None else float(mass_gamma)
    o.top_k_per_block = None if top_k_per_block is None else top_k_per_block.data_ptr()
    o.v = None if v is None else v.data_ptr()
    o.head_pattern = None if head_pattern is None else head_pattern.data_ptr()
    return o


def row_capacity(p: SpaParams) -> int:
    t = ctypes.c_int32()
    _check(load_library().spa_row_capacity(ctypes.byref(p), ctypes.byref(t)))
    return t.value


def workspace_bytes(p: SpaParams) -> int:
    n = ctypes.c_size_t()
    _check(load_library().spa_workspace_bytes(ctypes.byref(p), ctypes.byref(n)))
    return n.value


def _workspace(p: SpaParams, device):
    return torch.empty(workspace_bytes(p), dtype=torch.uint8, device=device)


def pool(q, k, block_size, seq_lens=None):
    """sparse_prefill_pool: returns (q_pooled, k_pooled) fp32 (blocks past a ragged entry's end are
    left as allocated)."""
    _dev_bf16(q, k)
    p = _params_from(q, k, block_size, 0, 1, 0, None, seq_lens=seq_lens)
    B, Hq, S, D = q.shape
    NB = -(-S // block_size)
    qp = torch.empty((B, Hq, NB, D), dtype=torch.float32, device=q.device)
    kp = torch.empty((B, k.shape[1], -(-k.shape[2] // block_size), D), dtype=torch.float32, device=q.device)
    _check(load_library().sparse_prefill_pool(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(qp), _ptr(kp), _stream(q)))
    return qp, kp


def value_norms(v, block_size):
    """sparse_prefill_value_norms: ln of the mean value-vector norm per key block, fp32 [B,Hkv,NB]."""
    _dev_bf16(v)
    B, Hkv, S, D = v.shape
    p = make_params(batch=B, n_q_heads=Hkv, n_kv_heads=Hkv, seq_len=S, head_dim=D, block_size=block_size,
                    n_sink_blocks=0, n_local_blocks=1, top_k_blocks=0, v=v)
    out = torch.empty((B, Hkv, -(-S // block_size)), dtype=torch.float32, device=v.device)
    _check(load_library().sparse_prefill_value_norms(ctypes.byref(p), _ptr(v), _ptr(out), _stream(v)))
    return out


def select(q, k, block_size, n_sink_blocks, n_local_blocks, top_k_blocks, softmax_scale=None,
           return_scores=False, workspace=None, top_k_per_block=None, v=None, stride_blocks=0,
           n_dense_q_blocks=0, head_pattern=None, stride_reach_blocks=0, group_shared=False, mass_gamma=None,
           seq_lens=None):
    """sparse_prefill_select; sparse_prefill_select_tpd when top_k_per_block (int32 [NB] device
    tensor) is given; sparse_prefill_select_stem when v is given (output-aware ranking, with or
    without a schedule); sparse_prefill_select_ex with head_pattern or mass_gamma (cumulative-mass
    budget).  Returns (block_idx, block_cnt[, scores])."""
    _dev_bf16(q, k)
    if v is not None:
        _dev_bf16(v)
    p = _params_from(q, k, block_size, n_sink_blocks, n_local_blocks, top_k_blocks, softmax_scale, v=v,
                     stride_blocks=stride_blocks, n_dense_q_blocks=n_dense_q_blocks,
                     stride_reach_blocks=stride_reach_blocks, group_shared=group_shared, seq_lens=seq_lens)
    B, Hq, S, _ = q.shape
    if group_shared:
        Hq = k.shape[1]                              # one list per KV head
    NB, T = -(-S // block_size), row_capacity(p)
    idx = torch.empty((B, Hq, NB, T), dtype=torch.int32, device=q.device)
    cnt = torch.empty((B, Hq, NB), dtype=torch.int32, device=q.device)
    NBk = -(-k.shape[2] // block_size)               # key blocks (more than NB with a KV prefix)
    sp = torch.empty((B, Hq, NB, NBk), dtype=torch.float32, device=q.device) if return_scores else None
    ws = _workspace(p, q.device) if workspace is None else workspace
    if head_pattern is not None or mass_gamma is not None:
        kr = None if top_k_per_block is None else _schedule(top_k_per_block, NB, q.device)
        o = _opts(kr, v, None if head_pattern is None else _head_pattern(head_pattern, Hq), mass_gamma)
        _check(load_library().sparse_prefill_select_ex(ctypes.byref(p), _ptr(q), _ptr(k), ctypes.byref(o), _ptr(idx),
                                                       _ptr(cnt), _ptr(sp), _ptr(ws), ws.numel(), _stream(q)))
    elif v is not None:
        kr = None if top_k_per_block is None else _schedule(top_k_per_block, NB, q.device)
        _check(load_library().sparse_prefill_select_stem(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(kr),
                                                         _ptr(idx), _ptr(cnt), _ptr(sp), _ptr(ws), ws.numel(),
                                                         _stream(q)))
    elif top_k_per_block is None:
        _check(load_library().sparse_prefill_select(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(idx), _ptr(cnt),
                                                    _ptr(sp), _ptr(ws), ws.numel(), _stream(q)))
    else:
        kr = _schedule(top_k_per_block, NB, q.device)
        _check(load_library().sparse_prefill_select_tpd(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(kr), _ptr(idx),
                                                        _ptr(cnt), _ptr(sp), _ptr(ws), ws.numel(), _stream(q)))
    return (idx, cnt, sp) if return_scores else (idx, cnt)


STATIC_SCRATCH_BYTES = 8 << 20


def select_static(q, k, block_size, n_sink_blocks, n_local_blocks, top_k_blocks, softmax_scale=None,
                  return_scores=False, group_shared=False, seq_lens=None, block_idx=None, block_cnt=None):
    """sparse_prefill_select_static: the plain select call on the library's own static scratch (no
    workspace).  block_idx / block_cnt may be passed in (a caller that must not allocate); otherwise
    they are made here.  Returns (block_idx, block_cnt[, scores])."""
    _dev_bf16(q, k)
    p = _params_from(q, k, block_size, n_sink_blocks, n_local_blocks, top_k_blocks, softmax_scale,
                     group_shared=group_shared, seq_lens=seq_lens)
    B, Hq, S, _ = q.shape
    if group_shared:
        Hq = k.shape[1]
    NB, T = -(-S // block_size), row_capacity(p)
    idx = torch.empty((B, Hq, NB, T), dtype=torch.int32, device=q.device) if block_idx is None else block_idx
    cnt = torch.empty((B, Hq, NB), dtype=torch.int32, device=q.device) if block_cnt is None else block_cnt
    if tuple(idx.shape) != (B, Hq, NB, T) or tuple(cnt.shape) != (B, Hq, NB) or idx.dtype != torch.int32 \
            or cnt.dtype != torch.int32 or not idx.is_contiguous() or not cnt.is_contiguous():
        raise TypeError("block_idx / block_cnt must be contiguous int32 [B,H,NB,T] / [B,H,NB]")
    NBk = -(-k.shape[2] // block_size)
    sp = torch.empty((B, Hq, NB, NBk), dtype=torch.float32, device=q.device) if return_scores else None
    _check(load_library().sparse_prefill_select_static(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(idx), _ptr(cnt), _ptr(sp),
                                                       _stream(q)))
    return (idx, cnt, sp) if return_scores else (idx, cnt)


def topk_from_scores(scores, n_sink_blocks, n_local_blocks, top_k_blocks, top_k_per_block=None,
                     stride_blocks=0, n_dense_q_blocks=0, head_pattern=None, stride_reach_blocks=0, mass_gamma=None,
                     seq_lens=None):
    """sparse_prefill_topk_from_scores (…_tpd with a schedule, …_ex with head_pattern or mass_gamma) on
    [B,Hq,NB,NB] fp32 device scores."""
    if scores.dtype != torch.float32 or not scores.is_cuda or not scores.is_contiguous():
        raise TypeError("expected contiguous fp32 scores on the GPU")
    B, Hq, NB, NBk = scores.shape                    # NBk > NB: a KV prefix of NBk - NB blocks
    p = make_params(batch=B, n_q_heads=Hq, n_kv_heads=Hq, seq_len=NB * 64, head_dim=64, block_size=64,
                    kv_prefix_len=(NBk - NB) * 64,
                    n_sink_blocks=n_sink_blocks, n_local_blocks=n_local_blocks, top_k_blocks=top_k_blocks,
                    stride_blocks=stride_blocks, n_dense_q_blocks=n_dense_q_blocks,
                    stride_reach_blocks=stride_reach_blocks, seq_lens=seq_lens)   # seq_lens in tokens of 64-token blocks
    T = row_capacity(p)
    idx = torch.empty((B, Hq, NB, T), dtype=torch.int32, device=scores.device)
    cnt = torch.empty((B, Hq, NB), dtype=torch.int32, device=scores.device)
    if head_pattern is not None or mass_gamma is not None:
        kr = None if top_k_per_block is None else _schedule(top_k_per_block, NB, scores.device)
        o = _opts(kr, None, None if head_pattern is None else _head_pattern(head_pattern, Hq), mass_gamma)
        _check(load_library().sparse_prefill_topk_from_scores_ex(ctypes.byref(p), _ptr(scores), ctypes.byref(o),
                                                                 _ptr(idx), _ptr(cnt), _stream(scores)))
    elif top_k_per_block is None:
        _check(load_library().sparse_prefill_topk_from_scores(ctypes.byref(p), _ptr(scores), _ptr(idx), _ptr(cnt),
                                                              _stream(scores)))
    else:
        kr = _schedule(top_k_per_block, NB, scores.device)
        _check(load_library().sparse_prefill_topk_from_scores_tpd(ctypes.byref(p), _ptr(scores), _ptr(kr),
                                                                  _ptr(idx), _ptr(cnt), _stream(scores)))
    return idx, cnt


def attn(q, k, v, block_idx, block_cnt, block_size, softmax_scale=None, return_lse=False, out=None,
         workspace=None, pattern=None, group_shared=False, seq_lens=None):
    """sparse_prefill_attn: returns out bf16 [B,Hq,S,D] (and lse fp32 [B,Hq,S]).
    pattern: optional (n_sink, n_local, top_k, stride_blocks, n_dense_q_blocks[, stride_reach_blocks]) the lists were made
    with; it only tells the library how uneven the rows are (scheduling hint)."""
    _dev_bf16(q, k, v)
    B, Hq, S, D = q.shape
    out = torch.empty((B, Hq, S, D), dtype=torch.bfloat16, device=q.device) if out is None else out
    T = block_idx.shape[-1]
    # the pattern fields only fix T here; the lists themselves carry the selection
    if pattern is None:
        p = _params_from(q, k, block_size, 0, 1, max(T - 1, 0), softmax_scale, v=v, out=out,
                         group_shared=group_shared, seq_lens=seq_lens)
    else:
        ns, nl, tk, stride, n_dense, *rest = pattern
        p = _params_from(q, k, block_size, ns, nl, tk, softmax_scale, v=v, out=out, stride_blocks=stride,
                         n_dense_q_blocks=n_dense, stride_reach_blocks=rest[0] if rest else 0,
                         group_shared=group_shared, seq_lens=seq_lens)
    if block_idx.shape[1] != (k.shape[1] if group_shared else Hq):
        raise TypeError("block_idx has the wrong number of heads for this call")
    if row_capacity(p) != T or block_idx.dtype != torch.int32 or block_cnt.dtype != torch.int32 \
            or not block_idx.is_contiguous() or not block_cnt.is_contiguous():
        raise TypeError("block_idx must be contiguous int32 [B,Hq,NB,T] with T <= NB")
    lse = torch.empty((B, Hq, S), dtype=torch.float32, device=q.device) if return_lse else None
    ws = _workspace(p, q.device) if workspace is None else workspace
    _check(load_library().sparse_prefill_attn(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(block_idx),
                                              _ptr(block_cnt), _ptr(out), _ptr(lse), _ptr(ws), ws.numel(),
                                              _stream(q)))
    return (out, lse) if return_lse else out


def transpose_v(v, block_size, vt=None, blocks_per_head=None, first_block=0, n_blocks=None, kv_prefix_len=0,
                seq_lens=None):
    """sparse_prefill_transpose_v: V [B,Hkv,Skv,D] -> vt [B,Hkv,blocks_per_head,D,Bs] bf16 (made here unless
    given), blocks first_block .. first_block + n_blocks - 1 (default: all).  With seq_lens (ragged batch),
    kv_prefix_len says how many of the Skv tokens are the prefix that every entry has in full."""
    _dev_bf16(v)
    B, Hkv, Skv, D = v.shape
    p = make_params(batch=B, n_q_heads=Hkv, n_kv_heads=Hkv, seq_len=Skv - kv_prefix_len, head_dim=D,
                    block_size=block_size, n_sink_blocks=0, n_local_blocks=1, top_k_blocks=0, v=v,
                    kv_prefix_len=kv_prefix_len, seq_lens=seq_lens)
    NBk = -(-Skv // block_size)
    bph = NBk if blocks_per_head is None else int(blocks_per_head)
    if vt is None:
        vt = torch.zeros((B, Hkv, bph, D, block_size), dtype=torch.bfloat16, device=v.device)
    if vt.dtype != torch.bfloat16 or not vt.is_cuda or not vt.is_contiguous() or tuple(vt.shape) != (B, Hkv, bph, D, block_size):
        raise TypeError("vt must be a contiguous bf16 device tensor [B,Hkv,blocks_per_head,D,Bs]")
    n = NBk - first_block if n_blocks is None else n_blocks
    _check(load_library().sparse_prefill_transpose_v(ctypes.byref(p), _ptr(v), _ptr(vt), bph, first_block, n, _stream(v)))
    return vt


def attn_vt(q, k, vt, block_idx, block_cnt, block_size, softmax_scale=None, return_lse=False, out=None,
            pattern=None, group_shared=False, seq_lens=None):
    """sparse_prefill_attn_vt: sparse_prefill_attn on a V^T the caller keeps (transpose_v); no workspace."""
    _dev_bf16(q, k, vt)
    B, Hq, S, D = q.shape
    out = torch.empty((B, Hq, S, D), dtype=torch.bfloat16, device=q.device) if out is None else out
    T = block_idx.shape[-1]
    if pattern is None:
        p = _params_from(q, k, block_size, 0, 1, max(T - 1, 0), softmax_scale, out=out, group_shared=group_shared,
                         seq_lens=seq_lens)
    else:
        ns, nl, tk, stride, n_dense, *rest = pattern
        p = _params_from(q, k, block_size, ns, nl, tk, softmax_scale, out=out, stride_blocks=stride,
                         n_dense_q_blocks=n_dense, stride_reach_blocks=rest[0] if rest else 0,
                         group_shared=group_shared, seq_lens=seq_lens)
    if vt.dim() != 5 or not vt.is_contiguous() or vt.shape[0] != B or vt.shape[1] != k.shape[1] \
            or tuple(vt.shape[3:]) != (D, block_size):
        raise TypeError("vt must be contiguous [B,Hkv,blocks_per_head,D,Bs]")
    if row_capacity(p) != T or block_idx.dtype != torch.int32 or block_cnt.dtype != torch.int32 \
            or not block_idx.is_contiguous() or not block_cnt.is_contiguous():
        raise TypeError("block_idx must be contiguous int32 [B,Hq,NB,T] with T <= NB")
    lse = torch.empty((B, Hq, S), dtype=torch.float32, device=q.device) if return_lse else None
    _check(load_library().sparse_prefill_attn_vt(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(vt), vt.shape[2], _ptr(block_idx),
                                                 _ptr(block_cnt), _ptr(out), _ptr(lse), _stream(q)))
    return (out, lse) if return_lse else out


def check_lists(q, k, block_idx, block_cnt, block_size, pattern=None, group_shared=False, seq_lens=None) -> int:
    """sparse_prefill_check_lists: the number of list rows that break the attention kernel's layout
    rules (0 = all well formed).  q, k only give the shape; pattern as in attn()."""
    B, Hq, S, D = q.shape
    T = block_idx.shape[-1]
    if pattern is None:
        p = _params_from(q, k, block_size, 0, 1, max(T - 1, 0), None, group_shared=group_shared, seq_lens=seq_lens)
    else:
        ns, nl, tk, stride, n_dense, *rest = pattern
        p = _params_from(q, k, block_size, ns, nl, tk, None, stride_blocks=stride, n_dense_q_blocks=n_dense,
                         stride_reach_blocks=rest[0] if rest else 0, group_shared=group_shared, seq_lens=seq_lens)
    if row_capacity(p) != T or block_idx.dtype != torch.int32 or block_cnt.dtype != torch.int32 \
            or not block_idx.is_contiguous() or not block_cnt.is_contiguous():
        raise TypeError("block_idx must be contiguous int32 [B,H,NB,T] with the call's row capacity")
    n_bad = torch.empty(1, dtype=torch.int32, device=block_idx.device)
    _check(load_library().sparse_prefill_check_lists(ctypes.byref(p), _ptr(block_idx), _ptr(block_cnt), _ptr(n_bad),
                                                     _stream(block_idx)))
    return int(n_bad.item())


def fused(q, k, v, block_size, n_sink_blocks, n_local_blocks, top_k_blocks, softmax_scale=None,
          return_lse=False, return_lists=False, workspace=None, out=None, top_k_per_block=None,
          output_aware=False, stride_blocks=0, n_dense_q_blocks=0, head_pattern=None, stride_reach_blocks=0,
          group_shared=False, mass_gamma=None, seq_lens=None):
    """sparse_prefill_fused (…_tpd with a schedule, …_stem with output_aware): select + attn on the
    current stream."""
    _dev_bf16(q, k, v)
    B, Hq, S, D = q.shape
    out = torch.empty((B, Hq, S, D), dtype=torch.bfloat16, device=q.device) if out is None else out
    p = _params_from(q, k, block_size, n_sink_blocks, n_local_blocks, top_k_blocks, softmax_scale, v=v, out=out,
                     stride_blocks=stride_blocks, n_dense_q_blocks=n_dense_q_blocks,
                     stride_reach_blocks=stride_reach_blocks, group_shared=group_shared, seq_lens=seq_lens)
    NB, T = -(-S // block_size), row_capacity(p)
    Hl = k.shape[1] if group_shared else Hq          # heads in the lists
    idx = torch.empty((B, Hl, NB, T), dtype=torch.int32, device=q.device) if return_lists else None
    cnt = torch.empty((B, Hl, NB), dtype=torch.int32, device=q.device) if return_lists else None
    lse = torch.empty((B, Hq, S), dtype=torch.float32, device=q.device) if return_lse else None
    ws = _workspace(p, q.device) if workspace is None else workspace
    if head_pattern is not None or mass_gamma is not None:
        kr = None if top_k_per_block is None else _schedule(top_k_per_block, NB, q.device)
        o = _opts(kr, v if output_aware else None, None if head_pattern is None else _head_pattern(head_pattern, Hl),
                  mass_gamma)
        _check(load_library().sparse_prefill_fused_ex(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), ctypes.byref(o),
                                                      _ptr(out), _ptr(lse), _ptr(idx), _ptr(cnt), _ptr(ws),
                                                      ws.numel(), _stream(q)))
    elif output_aware:
        kr = None if top_k_per_block is None else _schedule(top_k_per_block, NB, q.device)
        _check(load_library().sparse_prefill_fused_stem(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(kr),
                                                        _ptr(out), _ptr(lse), _ptr(idx), _ptr(cnt), _ptr(ws),
                                                        ws.numel(), _stream(q)))
    elif top_k_per_block is None:
        _check(load_library().sparse_prefill_fused(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse),
                                                   _ptr(idx), _ptr(cnt), _ptr(ws), ws.numel(), _stream(q)))
    else:
        kr = _schedule(top_k_per_block, NB, q.device)
        _check(load_library().sparse_prefill_fused_tpd(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(kr),
                                                       _ptr(out), _ptr(lse), _ptr(idx), _ptr(cnt), _ptr(ws),
                                                       ws.numel(), _stream(q)))
    res = [out]
    if return_lse:
        res.append(lse)
    if return_lists:
        res += [idx, cnt]
    return res[0] if len(res) == 1 else tuple(res)
