"""Seeded synthetic inputs for the sparse-prefill path.

This module holds only workload shapes and random-tensor recipes.  It contains
none of the method's arithmetic (no pooling, scoring, selection or attention)
and is the one piece of code shared by the HIP path's tests/bench and by the
CPU oracle's tests.

The tensors stand in for long-context prefill activations of 8B-class GQA
models (32 query / 8 KV heads, head_dim 128), the models the paper's sparse
attention section targets (Sec. 4.1.1, "Overall Framework"); the paper's own
workloads need datasets and weights that are not available here.

Every head of every tensor is drawn from its own generator seed, so a test can
materialise a single head of a 256K-token workload without generating the rest.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    seed: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    seq_len: int
    head_dim: int
    block_size: int
    n_sink_blocks: int
    n_local_blocks: int
    top_k_blocks: int
    n_hot_blocks: int = 0        # planted "hot" key blocks per KV head
    hot_gain: float = 3.0        # keys of a hot block += hot_gain * u_h
    drift: bool = False          # keys += (t / S) * w_h
    student_t_keys: bool = False  # keys ~ Student-t with 3 degrees of freedom

    @property
    def n_blocks(self) -> int:
        return self.seq_len // self.block_size

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def row_capacity(self) -> int:
        """T = min(NB, sink + local + topk): the width of one block-index row."""
        return min(self.n_blocks,
                   self.n_sink_blocks + self.n_local_blocks + self.top_k_blocks)

    @property
    def visited_pairs_per_head(self) -> int:
        t, nb = self.row_capacity, self.n_blocks
        return t * nb - t * (t - 1) // 2

    @property
    def visited_pairs(self) -> int:
        return self.batch * self.n_q_heads * self.visited_pairs_per_head

    @property
    def attn_flops(self) -> int:
        """4*Bs^2*D per visited (query block, key block) pair, diagonal counted full."""
        return 4 * self.block_size ** 2 * self.head_dim * self.visited_pairs

    @property
    def select_bytes(self) -> int:
        """Q and K read once, bf16."""
        return 2 * self.batch * (self.n_q_heads + self.n_kv_heads) * self.seq_len * self.head_dim

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


# The five workloads of the benchmark plan; index = config number.
WORKLOADS = (
    Workload("tiny_s512", 0, 1, 1, 1, 512, 64, 64, 1, 2, 2),
    Workload("s16k_b64", 1, 1, 32, 8, 16384, 128, 64, 1, 4, 16, n_hot_blocks=8),
    Workload("s32k_b128", 2, 1, 32, 8, 32768, 128, 128, 1, 2, 32, n_hot_blocks=16),
    Workload("s128k_b128", 3, 1, 32, 8, 131072, 128, 128, 1, 4, 64, n_hot_blocks=64, drift=True),
    Workload("s256k_b128", 4, 1, 40, 8, 262144, 128, 128, 2, 8, 96, n_hot_blocks=128,
             student_t_keys=True),
)


def workload(i: int) -> Workload:
    return WORKLOADS[i]


_TENSOR_ID = {"q": 1, "k": 2, "v": 3, "hot": 4, "u": 5, "w": 6}


def _gen(w: Workload, tensor: str, b: int, h: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(((w.seed * 1_000_003 + _TENSOR_ID[tensor]) * 10_007 + b) * 1_009 + h)
    return g


def _unit_vector(w: Workload, tensor: str, b: int, h: int) -> torch.Tensor:
    x = torch.randn(w.head_dim, generator=_gen(w, tensor, b, h), dtype=torch.float32)
    return x / x.norm()


def hot_blocks(w: Workload, b: int, kv_head: int) -> torch.Tensor:
    """Positions of the planted hot key blocks of one KV head (never a sink block)."""
    if w.n_hot_blocks == 0:
        return torch.empty(0, dtype=torch.int64)
    n_free = w.n_blocks - w.n_sink_blocks
    perm = torch.randperm(n_free, generator=_gen(w, "hot", b, kv_head))
    return perm[: min(w.n_hot_blocks, n_free)] + w.n_sink_blocks


def head_tensor(w: Workload, tensor: str, b: int, h: int) -> torch.Tensor:
    """One head of Q, K or V: [S, D] bf16 on the CPU."""
    assert tensor in ("q", "k", "v")
    shape = (w.seq_len, w.head_dim)
    x = torch.randn(shape, generator=_gen(w, tensor, b, h), dtype=torch.float32)
    if tensor == "k":
        if w.student_t_keys:
            g = _gen(w, "w", b, h)
            chi2 = torch.randn((3, w.seq_len, 1), generator=g, dtype=torch.float32).square().sum(0)
            x = x / (chi2 / 3.0).sqrt()
        if w.n_hot_blocks:
            u = _unit_vector(w, "u", b, h)
            xb = x.view(w.n_blocks, w.block_size, w.head_dim)
            xb[hot_blocks(w, b, h)] += w.hot_gain * u
        if w.drift:
            wv = _unit_vector(w, "w", b, h)
            pos = torch.arange(w.seq_len, dtype=torch.float32).unsqueeze(1) / float(w.seq_len)
            x = x + pos * wv
    return x.to(torch.bfloat16)


def make_qkv(w: Workload, device: str | torch.device = "cpu"):
    """Q [B,Hq,S,D], K and V [B,Hkv,S,D], bf16, contiguous, on `device`.

    Heads are generated one at a time on the CPU and copied into place so the
    fp32 staging never exceeds one head.
    """
    out = []
    for tensor, nh in (("q", w.n_q_heads), ("k", w.n_kv_heads), ("v", w.n_kv_heads)):
        t = torch.empty((w.batch, nh, w.seq_len, w.head_dim), dtype=torch.bfloat16, device=device)
        for b in range(w.batch):
            for h in range(nh):
                t[b, h].copy_(head_tensor(w, tensor, b, h))
        out.append(t)
    return tuple(out)


def decay_schedule(w: Workload, k_first: int | None = None, k_last: int | None = None) -> torch.Tensor:
    """A position-decaying top-k budget per query block, int32 [NB] on the CPU: k_first blocks for
    the first query block falling linearly to k_last for the last one (defaults: the workload's
    top_k and a quarter of it).  The paper's Token Position-Decay (Sec. 4.1.2, Fig. "Stem" (b))
    gives early positions the larger budget but prints no schedule; this one is a stand-in input."""
    k_first = w.top_k_blocks if k_first is None else k_first
    k_last = max(w.top_k_blocks // 4, 0) if k_last is None else k_last
    nb = w.n_blocks
    pos = torch.arange(nb, dtype=torch.float64) / max(nb - 1, 1)
    return torch.round(k_first + (k_last - k_first) * pos).to(torch.int32)


def sample_rows(w: Workload, n_random: int, seed: int = 0):
    """(b, h, i) rows for sampled parity at full size: the structural corner
    rows of a few heads plus seeded random ones."""
    nb, t = w.n_blocks, w.row_capacity
    corner = sorted({0, min(1, nb - 1), max(t - 2, 0), min(t - 1, nb - 1), min(t, nb - 1), nb // 2, nb - 1})
    rows = []
    for h in sorted({0, w.n_q_heads - 1}):
        rows += [(0, h, i) for i in corner]
    g = torch.Generator(device="cpu")
    g.manual_seed(977 * w.seed + seed + 13)
    for _ in range(n_random):
        b = int(torch.randint(w.batch, (1,), generator=g))
        h = int(torch.randint(w.n_q_heads, (1,), generator=g))
        i = int(torch.randint(nb, (1,), generator=g))
        rows.append((b, h, i))
    seen, uniq = set(), []
    for r in rows:
        if r not in seen:
            seen.add(r)
            uniq.append(r)
    return uniq
