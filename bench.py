#!/usr/bin/env python3
"""Benchmark of the sparse-prefill hot path on one MI355X.

A step is one pass of the whole path (pool -> score/top-k/merge -> block-sparse
attention) over one synthetic 131072-token batch (workload 3: 32 query / 8 KV
heads, head_dim 128, block 128, sink 1 + local 4 + top-k 64).  Inputs are
resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload N] [--no-cpu-baseline]
                    [--variant uniform|tpd|stem|strided|trishape|shared|mass] [--no-sample-power]

The line carries, under "power", the shader clock and socket power the driver reports in sysfs, sampled
from a side thread every 20 ms while the timed steps run (--no-sample-power leaves it out; a loop of two
seconds or more, e.g. --steps 150, gives the settled values).

--variant (default uniform = the headline) times the same workload under the other selection
rules the library has: a position-decaying budget (tpd), that plus the output-aware ranking
score (stem), strided static columns, a Tri-shape dense strip, group-shared lists, or a cumulative-mass
budget of 0.9 under the same count cap (mass); FLOPs are then counted on the block pairs the lists
actually hold.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E


def read_traffic_note(kernel: str, workload: str):
    """(HBM bytes per launch of `kernel` at `workload`, where the figure comes from) out of the committed
    counter summaries, or (None, None): it is a recorded measurement of an earlier run of the same
    command under rocprofv3 --pmc, not a measurement of this run."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    if not os.path.exists(path):
        return None, None
    for line in open(path):
        parts = line.split()
        if len(parts) >= 2 and parts[0] == kernel:
            try:
                return float(parts[1]), "recorded: profiles/" + os.path.basename(path) + " (rocprofv3 --pmc runs of this command)"
            except ValueError:
                return None, None
    return None, None


class PowerSampler:
    """Shader clock (pp_dpm_sclk, the level marked current) and socket power (hwmon power1_input or
    power1_average) of the first GPU that exposes them in sysfs, read every `period` seconds."""

    def __init__(self, period=0.02, root="/sys/class/drm"):
        import glob
        self.period, self.clock, self.power, self._stop, self._thread = period, [], [], False, None
        self.sclk = self.pwr = None
        for dev in sorted(glob.glob(os.path.join(root, "card*", "device"))):
            sclk = os.path.join(dev, "pp_dpm_sclk")
            pw = [f for n in ("power1_input", "power1_average") for f in glob.glob(os.path.join(dev, "hwmon", "hwmon*", n))]
            if os.access(sclk, os.R_OK) and pw:
                self.sclk, self.pwr = sclk, pw[0]
                break

    def _read(self):
        try:
            for line in open(self.sclk):
                if "*" in line:
                    self.clock.append(float(line.split(":")[1].lower().split("mhz")[0]))
                    break
            self.power.append(float(open(self.pwr).read()) * 1e-6)
        except (OSError, ValueError, IndexError):
            pass

    def _run(self):
        while not self._stop:
            self._read()
            time.sleep(self.period)

    def start(self):
        import threading
        if self.sclk is None:
            return
        self._thread = threading.Thread(target=self._run, daemon=True)
        self._thread.start()

    def stop(self):
        self._stop = True
        if self._thread is not None:
            self._thread.join()

    @staticmethod
    def _stats(xs):
        if not xs:
            return None
        xs = sorted(xs)
        return {"min": xs[0], "p10": xs[len(xs) // 10], "median": xs[len(xs) // 2], "max": xs[-1], "samples": len(xs)}

    def summary(self):
        return {"shader_clock_mhz": self._stats(self.clock), "socket_power_w": self._stats(self.power),
                "source": f"{self.sclk} (current level), {self.pwr}", "period_s": self.period}


def cpu_baseline(w, q, k, v, idx, cnt, n_rows):
    """The oracle, as it stands, on a bounded sample of the same workload."""
    from oracle import oracle
    from paper_2602_21233_amd import inputs
    t0 = time.perf_counter()
    oracle.select(q, k, w.block_size, w.n_sink_blocks, w.n_local_blocks, w.top_k_blocks)
    t_select = time.perf_counter() - t0
    rows = inputs.sample_rows(w, n_rows, seed=1)[:n_rows]
    t0 = time.perf_counter()
    oracle.attn(q, k, v, idx, cnt, w.block_size, rows=rows)
    t_attn = time.perf_counter() - t0
    pairs = sum(int(cnt[b, h, i]) for (b, h, i) in rows)
    frac = len(rows) / float(w.batch * w.n_q_heads * w.n_blocks)
    flops = 4.0 * w.block_size ** 2 * w.head_dim * pairs
    t = t_attn + t_select * frac
    return {
        "value": flops / t / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
        "sample": f"attention on {len(rows)} of {w.batch * w.n_q_heads * w.n_blocks} query-block rows "
                  f"({pairs} visited pairs, {t_attn:.1f} s) + full select stage ({t_select:.1f} s) pro-rated",
        "extrapolated_ms_per_step": (t_attn / frac + t_select) * 1e3,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-rows", type=int, default=1200)
    ap.add_argument("--cold", action="store_true",
                    help="overwrite a 1-GiB scratch buffer before every step (cold caches; for the small "
                         "workloads); ms_per_step then comes from the events, not the wall clock")
    ap.add_argument("--no-sample-power", action="store_true",
                    help="do not sample the reported shader clock and socket power during the timed steps")
    ap.add_argument("--variant", choices=("uniform", "tpd", "stem", "strided", "trishape", "shared", "mass"),
                    default="uniform")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (heads shard across GPUs with no exchange; "
              "no multi-GPU figure is produced). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2602_21233_amd as spa
    from paper_2602_21233_amd import binding, inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    spa.load_library()
    w = inputs.workload(args.workload)
    q, k, v = inputs.make_qkv(w)
    dq, dk, dv = q.cuda(), k.cuda(), v.cuda()
    Bs, ns, nl, tk = w.block_size, w.n_sink_blocks, w.n_local_blocks, w.top_k_blocks
    p = binding.make_params(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, seq_len=w.seq_len,
                            head_dim=w.head_dim, block_size=Bs, n_sink_blocks=ns, n_local_blocks=nl,
                            top_k_blocks=tk, q=dq, k=dk, v=dv, out=dq)
    ws = torch.empty(spa.workspace_bytes(p), dtype=torch.uint8, device="cuda")
    out = torch.empty_like(dq)

    sel_kw, pat_kw = {}, {}
    if args.variant in ("tpd", "stem"):
        sel_kw["top_k_per_block"] = inputs.decay_schedule(w).cuda()
    if args.variant == "stem":
        sel_kw["v"] = dv
    if args.variant == "mass":
        sel_kw["mass_gamma"] = 0.9
    if args.variant == "strided":
        pat_kw = dict(stride_blocks=16)
    if args.variant == "trishape":
        pat_kw = dict(n_dense_q_blocks=8)
    shared = args.variant == "shared"
    if shared:
        sel_kw["group_shared"] = True
    if pat_kw or shared:
        p = binding.make_params(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, seq_len=w.seq_len,
                                head_dim=w.head_dim, block_size=Bs, n_sink_blocks=ns, n_local_blocks=nl,
                                top_k_blocks=tk, q=dq, k=dk, v=dv, out=dq, lists_per_kv_head=shared, **pat_kw)
        ws = torch.empty(spa.workspace_bytes(p), dtype=torch.uint8, device="cuda")

    pattern = (ns, nl, tk, pat_kw.get("stride_blocks", 0), pat_kw.get("n_dense_q_blocks", 0))

    flush = torch.empty(1 << 30, dtype=torch.uint8, device="cuda") if args.cold else None

    # V^T of the attention stage: the buffer sparse_prefill_attn would take from the workspace
    vt = torch.empty((w.batch, w.n_kv_heads, w.n_blocks, w.head_dim, Bs), dtype=torch.bfloat16, device="cuda")

    def step(events=None):
        # the same launches sparse_prefill_fused makes (select; then the two halves of
        # sparse_prefill_attn: V transpose and attention kernel), split so that the attention
        # kernel alone can be bracketed by events on its own stream
        if flush is not None:
            flush.fill_(1)
        if events:
            events[0].record()
        idx, cnt = spa.select(dq, dk, Bs, ns, nl, tk, workspace=ws, **sel_kw, **pat_kw)
        if events:
            events[1].record()
        spa.transpose_v(dv, Bs, vt=vt)
        if events:
            events[2].record()
        spa.attn_vt(dq, dk, vt, idx, cnt, Bs, out=out, pattern=pattern, group_shared=shared)
        if events:
            events[3].record()
        return idx, cnt

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    sampler = None if args.no_sample_power else PowerSampler()
    if sampler:
        sampler.start()
    t0 = time.perf_counter()
    for s in range(args.steps):
        idx, cnt = step(evs[s])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    if sampler:
        sampler.stop()
    ms_step = wall * 1e3 / args.steps
    if args.cold:
        ms_step = sum(e[0].elapsed_time(e[3]) for e in evs) / args.steps
    sel_ms = sorted(e[0].elapsed_time(e[1]) for e in evs)
    att_ms = sorted(e[1].elapsed_time(e[3]) for e in evs)          # attention stage: V transpose + attention kernel
    tv_ms = sorted(e[1].elapsed_time(e[2]) for e in evs)
    ker_ms = sorted(e[2].elapsed_time(e[3]) for e in evs)          # the attention kernel alone
    sel_avg, att_avg = sum(sel_ms) / len(sel_ms), sum(att_ms) / len(att_ms)
    ker_avg = sum(ker_ms) / len(ker_ms)

    # the one-call entry point (select + attention in one C call), timed the same way
    fused_ms = None
    if args.variant == "uniform":
        fev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
        for a, b in fev:
            if flush is not None:
                flush.fill_(1)
            a.record()
            spa.fused(dq, dk, dv, Bs, ns, nl, tk, workspace=ws, out=out)
            b.record()
        torch.cuda.synchronize()
        f = sorted(a.elapsed_time(b) for a, b in fev)
        fused_ms = {"avg": sum(f) / len(f), "p10": f[len(f) // 10], "p50": f[len(f) // 2], "p90": f[(len(f) * 9) // 10]}

    # the output-aware score reads V once more (2 bytes per element)
    select_bytes = w.select_bytes + (2 * w.batch * w.n_kv_heads * w.seq_len * w.head_dim if args.variant == "stem" else 0)
    visited_pairs = int(cnt.sum().item()) * (w.group if shared else 1)        # what the GPU's own lists hold
    if args.variant == "uniform" and visited_pairs != w.visited_pairs:
        print(f"bench.py: the lists hold {visited_pairs} block pairs, the closed form says {w.visited_pairs}", file=sys.stderr)
        sys.exit(1)
    flops = 4.0 * Bs * Bs * w.head_dim * visited_pairs
    achieved = flops / (ker_avg * 1e-3) / 1e12
    traffic, traffic_source = read_traffic_note("attn_kernel", w.name) if args.variant == "uniform" else (None, None)
    # the launcher's choice: two heads per workgroup when the group shares its lists; with one head per
    # workgroup, blocks of 64 tokens take the chunked kernel
    heads_per_wg = 2 if shared and w.group % 2 == 0 else 1
    kernel_name = f"{'attn_chunked_kernel' if Bs == 64 and heads_per_wg == 1 else 'attn_kernel'}<{Bs},{w.head_dim},{heads_per_wg}>"
    result = {
        "metric": f"sparse prefill attention effective TFLOP/s on visited blocks (select + attention), "
                  f"{w.seq_len // 1024}K tokens" + ("" if args.variant == "uniform" else f", variant {args.variant}"),
        "value": flops / (ms_step * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads,
                   "seq_len": w.seq_len, "head_dim": w.head_dim, "block_size": Bs, "sink_blocks": ns,
                   "local_blocks": nl, "top_k_blocks": tk, "visited_pairs": visited_pairs,
                   "flops_per_step": flops, "variant": args.variant},
        "select_ms": {"avg": sel_avg, "p10": sel_ms[len(sel_ms) // 10], "p50": sel_ms[len(sel_ms) // 2],
                      "p90": sel_ms[(len(sel_ms) * 9) // 10]},
        "attn_ms": {"avg": att_avg, "p10": att_ms[len(att_ms) // 10], "p50": att_ms[len(att_ms) // 2],
                    "p90": att_ms[(len(att_ms) * 9) // 10]},
        "transpose_v_ms": {"avg": sum(tv_ms) / len(tv_ms), "p50": tv_ms[len(tv_ms) // 2]},
        "fused_ms": fused_ms, "caches": "cold" if args.cold else "warm",
        "select_hbm": {"achieved": select_bytes / (sel_avg * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                       "frac": select_bytes / (sel_avg * 1e-3) / 1e9 / PEAK_HBM_GBS,
                       "bytes": select_bytes},
        "roofline": {"bound": "mfma", "kernel": kernel_name, "achieved": achieved, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
                     "avg_ms": ker_avg, "median_ms": ker_ms[len(ker_ms) // 2], "min_ms": ker_ms[0],
                     "stage_frac": flops / (att_avg * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                     "traffic": traffic, "traffic_unit": "bytes/launch", "traffic_source": traffic_source,
                     "timed": "events around the attention kernel's launch on its stream (sparse_prefill_attn_vt); the V transpose "
                              "that precedes it in sparse_prefill_attn is timed apart (attn_ms is the two together, "
                              "stage_frac the fraction on that time)"},
    }
    if sampler:
        result["power"] = sampler.summary()
    if not args.no_cpu_baseline and args.variant == "uniform":
        result["cpu_baseline"] = cpu_baseline(w, q, k, v, idx.cpu(), cnt.cpu(), args.cpu_rows)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
