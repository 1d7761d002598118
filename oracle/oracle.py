"""ctypes front end of the CPU oracle (oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg import this.
It shares nothing with the HIP library or its binding.  Tensors are torch CPU
tensors; bf16 inputs are passed as their bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile oracle.c with gcc.  No -march (the .so must run on another host),
    no fast-math, no fp contraction: the arithmetic is what the source says."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, f32, vp = ctypes.c_int64, ctypes.c_float, ctypes.c_void_p
        lib.oracle_pool.argtypes = [vp, i64, i64, i64, i64, vp]
        lib.oracle_scores.argtypes = [vp, vp, i64, i64, i64, i64, i64, i64, f32, vp]
        lib.oracle_topk.argtypes = [vp, i64, i64, i64, i64, i64, i64, vp, i64, i64, i64, vp, i64, vp, vp]
        lib.oracle_topk_mass.argtypes = [vp, i64, i64, i64, i64, i64, i64, vp, i64, i64, i64, vp, i64, ctypes.c_double, vp, vp]
        lib.oracle_mass_weights.argtypes = [vp, i64, i64, i64, vp]
        lib.oracle_row_capacity.argtypes = [i64] * 7
        lib.oracle_row_capacity.restype = ctypes.c_int64
        lib.oracle_vnorm.argtypes = [vp, i64, i64, i64, i64, vp]
        lib.oracle_scores_oam.argtypes = [vp, vp, i64, i64, i64, i64, i64]
        lib.oracle_attn.argtypes = [vp, vp, vp, i64, i64, i64, i64, i64, i64, i64, i64, f32,
                                    vp, vp, vp, i64, vp, vp]
        for f in (lib.oracle_pool, lib.oracle_scores, lib.oracle_topk, lib.oracle_attn,
                  lib.oracle_num_threads, lib.oracle_vnorm, lib.oracle_scores_oam, lib.oracle_topk_mass,
                  lib.oracle_mass_weights):
            f.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def default_scale(head_dim: int) -> float:
    """1/sqrt(D) evaluated in fp32 (the value both sides use when none is given)."""
    return float(np.float32(1.0) / np.sqrt(np.float32(head_dim)))


def row_capacity(n_blocks: int, ns: int, nl: int, k: int, stride: int = 0, n_dense: int = 0, reach: int = 0) -> int:
    return int(_load().oracle_row_capacity(n_blocks, ns, nl, k, stride, n_dense, reach))


def _bits(x: torch.Tensor) -> torch.Tensor:
    assert x.dtype == torch.bfloat16 and x.device.type == "cpu"
    return x.contiguous().view(torch.int16)


def _check(rc: int, what: str):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def pool(x: torch.Tensor, block_size: int) -> torch.Tensor:
    """x [B,H,S,D] bf16 -> [B,H,S/Bs,D] fp32 block means."""
    B, H, S, D = x.shape
    xb = _bits(x)
    out = torch.empty((B, H, -(-S // block_size), D), dtype=torch.float32)
    _check(_load().oracle_pool(xb.data_ptr(), B * H, S, D, block_size, out.data_ptr()), "pool")
    return out


def scores(qp: torch.Tensor, kp: torch.Tensor, scale: float) -> torch.Tensor:
    """qp [B,Hq,NBq,D], kp [B,Hkv,NBk,D] fp32 -> [B,Hq,NBq,NBk] fp32 (j > i + NBk - NBq: -inf).
    NBk > NBq is a KV prefix: the query blocks are the last NBq of the NBk blocks."""
    B, Hq, NB, D = qp.shape
    Hkv, NBk = kp.shape[1], kp.shape[2]
    qp, kp = qp.contiguous(), kp.contiguous()
    assert qp.dtype == torch.float32 and kp.dtype == torch.float32
    sp = torch.empty((B, Hq, NB, NBk), dtype=torch.float32)
    _check(_load().oracle_scores(qp.data_ptr(), kp.data_ptr(), B, Hq, Hkv, NB, NBk, D, scale,
                                 sp.data_ptr()), "scores")
    return sp


def vnorm(v: torch.Tensor, block_size: int) -> torch.Tensor:
    """v [B,Hkv,S,D] bf16 -> [B,Hkv,S/Bs] fp32: mean L2 norm of each block's value vectors."""
    B, H, S, D = v.shape
    vb = _bits(v)
    out = torch.empty((B, H, -(-S // block_size)), dtype=torch.float32)
    _check(_load().oracle_vnorm(vb.data_ptr(), B * H, S, D, block_size, out.data_ptr()), "vnorm")
    return out


def scores_oam(sp: torch.Tensor, vn: torch.Tensor) -> torch.Tensor:
    """Output-aware scores: sp[b,h,i,j] + ln vn[b,h/G,j] for j <= i (a copy; j > i untouched)."""
    B, Hq, NB, NBk = sp.shape
    Hkv = vn.shape[1]
    out = sp.contiguous().clone()
    vn = vn.contiguous()
    assert out.dtype == torch.float32 and vn.dtype == torch.float32 and vn.shape == (B, Hkv, NBk)
    _check(_load().oracle_scores_oam(out.data_ptr(), vn.data_ptr(), B, Hq, Hkv, NB, NBk), "scores_oam")
    return out


def mass_weights(sp: torch.Tensor) -> torch.Tensor:
    """Integer softmax weights of the cumulative-mass budget: sp [B,Hq,NBq,NBk] fp32 -> int64
    [B,Hq,NBq,NBk], W ~ 2^19 exp(score - row max) for the causal blocks, 0 beyond."""
    B, Hq, NB, NBk = sp.shape
    sp = sp.contiguous()
    assert sp.dtype == torch.float32
    w = torch.empty((B, Hq, NB, NBk), dtype=torch.int32)
    _check(_load().oracle_mass_weights(sp.data_ptr(), B * Hq, NB, NBk, w.data_ptr()), "mass_weights")
    return w.to(torch.int64) & 0xffffffff


def topk(sp: torch.Tensor, ns: int, nl: int, k: int, k_per_row: torch.Tensor | None = None,
         stride: int = 0, n_dense: int = 0, head_pattern: torch.Tensor | None = None, reach: int = 0,
         gamma: float | None = None):
    """sp [B,Hq,NBq,NBk] fp32 -> idx [B,Hq,NBq,T] int32 (pad -1), cnt [B,Hq,NBq] int32; NBk > NBq
    is a KV prefix of NBk - NBq blocks (pattern and capacity then refer to positions in NBk).
    k_per_row: optional [NB] int32 position-dependent budget (clamped to [0, k]).
    stride / n_dense: strided static columns and the dense bottom strip of the Tri-shape.
    head_pattern: optional [Hq,3] int32 (n_sink, n_local, top_k) per query head; ns, nl, k are
    then the maxima.
    gamma: optional cumulative-mass budget in [0, 1]: a row stops taking candidates once the selected
    blocks hold that fraction of its block-level softmax mass (count budgets stay as caps)."""
    B, Hq, NB, NBk = sp.shape
    sp = sp.contiguous()
    assert sp.dtype == torch.float32
    T = row_capacity(NBk, ns, nl, k, stride, n_dense, reach)
    idx = torch.empty((B, Hq, NB, T), dtype=torch.int32)
    cnt = torch.empty((B, Hq, NB), dtype=torch.int32)
    kr_ptr = None
    if k_per_row is not None:
        k_per_row = k_per_row.to(torch.int32).contiguous()
        assert k_per_row.shape == (NB,) and k_per_row.device.type == "cpu"
        kr_ptr = k_per_row.data_ptr()
    hp_ptr = None
    if head_pattern is not None:
        head_pattern = head_pattern.to(torch.int32).contiguous()
        assert head_pattern.shape == (Hq, 3) and head_pattern.device.type == "cpu"
        hp_ptr = head_pattern.data_ptr()
    if gamma is None:
        _check(_load().oracle_topk(sp.data_ptr(), B * Hq, NB, NBk, ns, nl, k, kr_ptr, stride, n_dense, reach, hp_ptr, Hq,
                                   idx.data_ptr(), cnt.data_ptr()), "topk")
    else:
        # the budget is stated as an fp32 number, like the library's parameter
        _check(_load().oracle_topk_mass(sp.data_ptr(), B * Hq, NB, NBk, ns, nl, k, kr_ptr, stride, n_dense, reach, hp_ptr,
                                        Hq, float(np.float32(gamma)), idx.data_ptr(), cnt.data_ptr()), "topk_mass")
    return idx, cnt


def select(q: torch.Tensor, k: torch.Tensor, block_size: int, ns: int, nl: int, topk_blocks: int,
           scale: float | None = None, k_per_row: torch.Tensor | None = None, v: torch.Tensor | None = None,
           stride: int = 0, n_dense: int = 0, head_pattern: torch.Tensor | None = None, reach: int = 0,
           group_shared: bool = False, gamma: float | None = None):
    """Pool, score, top-k, merge.  Returns (idx, cnt, sp, qp, kp).  With v the ranking score is
    the output-aware one (scores_oam) and sp is that score.

    group_shared: one list per KV head, shared by the G query heads of its group (a variant the
    paper's per-head metadata allows; reading: the group is ranked by the mean of its heads'
    pooled scores, i.e. by the score of the group-mean pooled query).  idx/cnt/sp then have
    n_kv_heads in the head axis and qp is the group mean [B,Hkv,NB,D]."""
    scale = default_scale(q.shape[-1]) if scale is None else scale
    qp, kp = pool(q, block_size), pool(k, block_size)
    if group_shared:
        B, Hq, NB, D = qp.shape
        Hkv = kp.shape[1]
        qp = qp.view(B, Hkv, Hq // Hkv, NB, D).double().mean(2).float()
    sp = scores(qp, kp, scale)
    if v is not None:
        sp = scores_oam(sp, vnorm(v, block_size))
    idx, cnt = topk(sp, ns, nl, topk_blocks, k_per_row, stride, n_dense, head_pattern, reach, gamma)
    return idx, cnt, sp, qp, kp


def attn(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, idx: torch.Tensor, cnt: torch.Tensor,
         block_size: int, scale: float | None = None, rows=None):
    """Block-sparse causal attention.  rows=None: out [B,Hq,S,D], lse [B,Hq,S];
    rows=[(b,h,i),...]: out [n,Bs,D], lse [n,Bs].  fp32 results of fp64 math."""
    B, Hq, S, D = q.shape
    Hkv, Skv = k.shape[1], k.shape[2]            # Skv > S: the queries are the last S tokens (KV prefix)
    T = idx.shape[-1]
    scale = default_scale(D) if scale is None else scale
    qb, kb, vb = _bits(q), _bits(k), _bits(v)
    idx = idx.contiguous().to(torch.int32)
    cnt = cnt.contiguous().to(torch.int32)
    if rows is None:
        n = B * Hq * (-(-S // block_size))
        out = torch.empty((B, Hq, S, D), dtype=torch.float32)
        lse = torch.empty((B, Hq, S), dtype=torch.float32)
        rows_ptr = None
    else:
        rows_t = torch.tensor(rows, dtype=torch.int32).reshape(-1, 3).contiguous()
        n = rows_t.shape[0]
        out = torch.empty((n, block_size, D), dtype=torch.float32)
        lse = torch.empty((n, block_size), dtype=torch.float32)
        rows_ptr = rows_t.data_ptr()
    _check(_load().oracle_attn(qb.data_ptr(), kb.data_ptr(), vb.data_ptr(), B, Hq, Hkv, S, Skv, D,
                               block_size, T, scale, idx.data_ptr(), cnt.data_ptr(), rows_ptr, n,
                               out.data_ptr(), lse.data_ptr()), "attn")
    return out, lse


# ---- ragged batches: every entry is a batch-1 problem of its own length ---------------------------
def select_ragged(q: torch.Tensor, k: torch.Tensor, seq_lens, block_size: int, ns: int, nl: int, topk_blocks: int,
                  **kw):
    """Entry b has seq_lens[b] query tokens and P + seq_lens[b] key tokens (P = k.shape[2] - q.shape[2],
    a KV prefix common to all entries); q, k keep their padded shapes.  Each entry is selected by a
    batch-1 call of select() on its own slice.  Returns padded (idx [B,H,NB,T], cnt [B,H,NB]) with
    T of the padded call; rows past an entry's last block have count 0 and -1 entries."""
    B, Hq, S, _ = q.shape
    P = k.shape[2] - S
    NB = -(-S // block_size)
    NBk = -(-(P + S) // block_size)
    Hl = k.shape[1] if kw.get("group_shared") else Hq
    T = row_capacity(NBk, ns, nl, topk_blocks, kw.get("stride", 0), kw.get("n_dense", 0), kw.get("reach", 0))
    idx = torch.full((B, Hl, NB, T), -1, dtype=torch.int32)
    cnt = torch.zeros((B, Hl, NB), dtype=torch.int32)
    for b in range(B):
        n = int(seq_lens[b])
        if n <= 0:
            continue
        kw_b = dict(kw)
        if kw_b.get("v") is not None:
            kw_b["v"] = kw_b["v"][b:b + 1, :, :P + n]
        if kw_b.get("k_per_row") is not None:
            kw_b["k_per_row"] = kw_b["k_per_row"][:-(-n // block_size)]
        i_b, c_b, *_ = select(q[b:b + 1, :, :n], k[b:b + 1, :, :P + n], block_size, ns, nl, topk_blocks, **kw_b)
        idx[b, :, :i_b.shape[2], :i_b.shape[3]] = i_b[0]
        cnt[b, :, :c_b.shape[2]] = c_b[0]
    return idx, cnt


def attn_ragged(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, idx: torch.Tensor, cnt: torch.Tensor, seq_lens,
                block_size: int, scale: float | None = None):
    """Attention of every entry on its own slice with its own lists.  Returns out [B,Hq,S,D] and
    lse [B,Hq,S] fp32, NaN where an entry has no token."""
    B, Hq, S, D = q.shape
    P = k.shape[2] - S
    out = torch.full((B, Hq, S, D), float("nan"), dtype=torch.float32)
    lse = torch.full((B, Hq, S), float("nan"), dtype=torch.float32)
    for b in range(B):
        n = int(seq_lens[b])
        if n <= 0:
            continue
        nb = -(-n // block_size)
        o_b, l_b = attn(q[b:b + 1, :, :n], k[b:b + 1, :, :P + n], v[b:b + 1, :, :P + n], idx[b:b + 1, :, :nb],
                        cnt[b:b + 1, :, :nb], block_size, scale)
        out[b, :, :n] = o_b[0]
        lse[b, :, :n] = l_b[0]
    return out, lse
