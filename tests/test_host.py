"""Host-side checks that need neither a GPU nor the oracle: the workload table against the
figures of the benchmark plan, the seeded input recipe, and bench.py's refusal of more than one GPU."""
import os
import subprocess
import sys

import pytest
import torch

from paper_2602_21233_amd import inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# (row capacity T, visited pairs per head, total pairs, select bytes) per workload: counted here by
# brute force over the rows (row i of the plain A-shape visits min(i + 1, T) blocks)
PLAN = {
    0: (5, 30, 30, 131_072),
    1: (21, 5_166, 165_312, 167_772_160),
    2: (35, 8_365, 267_680, 335_544_320),
    3: (69, 68_310, 2_185_920, 1_342_177_280),
    4: (106, 211_523, 8_460_920, 3_221_225_472),
}


@pytest.mark.parametrize("n", sorted(PLAN))
def test_workload_table_matches_the_plan(n):
    w = inputs.workload(n)
    T, per_head, total, sel_bytes = PLAN[n]
    assert w.seed == n and w.row_capacity == T
    brute = sum(min(i + 1, T) for i in range(w.n_blocks))
    assert brute == per_head == w.visited_pairs_per_head
    assert w.visited_pairs == total == per_head * w.batch * w.n_q_heads
    assert w.attn_flops == 4 * w.block_size ** 2 * w.head_dim * total
    assert w.select_bytes == sel_bytes


def test_headline_flops_figure():
    assert abs(inputs.workload(3).attn_flops - 1.834e13) < 0.001e13
    assert abs(inputs.workload(4).attn_flops - 7.10e13) < 0.01e13


def test_inputs_are_seeded_and_per_head():
    w = inputs.workload(1).scaled(seq_len=1024, n_q_heads=4, n_kv_heads=2)
    q1, k1, v1 = inputs.make_qkv(w)
    q2, k2, v2 = inputs.make_qkv(w)
    assert q1.dtype == torch.bfloat16 and q1.shape == (1, 4, 1024, 128) and k1.shape == v1.shape == (1, 2, 1024, 128)
    assert torch.equal(q1, q2) and torch.equal(k1, k2) and torch.equal(v1, v2)
    # a single head can be drawn without the rest, and heads differ
    assert torch.equal(inputs.head_tensor(w, "k", 0, 1), k1[0, 1])
    assert not torch.equal(k1[0, 0], k1[0, 1]) and not torch.equal(q1[0, 0], q1[0, 1])
    # another seed gives other tensors
    assert not torch.equal(inputs.make_qkv(w.scaled(seed=7))[0], q1)


def test_hot_blocks_carry_the_planted_direction():
    """Keys of a hot block are shifted by hot_gain * u_h (a unit vector per KV head): their mean along
    the block stands out by ~hot_gain in norm against ~sqrt(D / Bs) for an ordinary block."""
    w = inputs.workload(1).scaled(seq_len=4096, n_q_heads=4, n_kv_heads=2)
    hot = inputs.hot_blocks(w, 0, 1)
    assert len(hot) == w.n_hot_blocks == 8 and len(set(hot.tolist())) == 8
    assert hot.min().item() >= w.n_sink_blocks and hot.max().item() < w.n_blocks
    k = inputs.head_tensor(w, "k", 0, 1).float().view(w.n_blocks, w.block_size, w.head_dim)
    norms = k.mean(dim=1).norm(dim=1)
    is_hot = torch.zeros(w.n_blocks, dtype=torch.bool)
    is_hot[hot] = True
    assert norms[is_hot].min().item() > 2.5 and norms[~is_hot].max().item() < 2.2
    # all hot blocks of a head share the direction
    means = k.mean(dim=1)[is_hot]
    cos = torch.nn.functional.cosine_similarity(means[:1], means[1:], dim=1)
    assert cos.min().item() > 0.7


def test_decay_schedule_endpoints_and_monotone():
    w = inputs.workload(3)
    s = inputs.decay_schedule(w)
    assert s.dtype == torch.int32 and s.shape == (w.n_blocks,)
    assert s[0].item() == 64 and s[-1].item() == 16
    assert (s[1:] <= s[:-1]).all()


def test_sample_rows_hold_the_corner_rows():
    w = inputs.workload(3)
    rows = inputs.sample_rows(w, 50)
    T, NB = w.row_capacity, w.n_blocks
    got = {i for (_, h, i) in rows if h == 0}
    assert {0, T - 1, T, NB - 1} <= got
    assert all(0 <= b < w.batch and 0 <= h < w.n_q_heads and 0 <= i < NB for b, h, i in rows)
    assert rows == inputs.sample_rows(w, 50)


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_power_sampler_reads_the_current_clock_level_and_the_socket_power(tmp_path):
    """bench.py's side-thread sampler on a stand-in for the driver's sysfs files: the clock is the level marked
    current in pp_dpm_sclk, the power is hwmon's power1_input in microwatts; a GPU without the files gives None."""
    import importlib.util
    import time
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    dev = tmp_path / "card0" / "device"
    (dev / "hwmon" / "hwmon3").mkdir(parents=True)
    (dev / "pp_dpm_sclk").write_text("0: 500Mhz\n1: 1496Mhz *\n2: 2400Mhz\n")
    (dev / "hwmon" / "hwmon3" / "power1_input").write_text("1340000000\n")
    s = bench.PowerSampler(period=0.005, root=str(tmp_path))
    s.start()
    time.sleep(0.05)
    (dev / "pp_dpm_sclk").write_text("0: 500Mhz *\n1: 1496Mhz\n2: 2400Mhz\n")
    time.sleep(0.05)
    s.stop()
    out = s.summary()
    assert out["shader_clock_mhz"]["max"] == 1496.0 and out["shader_clock_mhz"]["min"] == 500.0
    assert out["socket_power_w"]["median"] == 1340.0 and out["socket_power_w"]["samples"] >= 4
    empty = bench.PowerSampler(root=str(tmp_path / "nothing"))
    empty.start()
    empty.stop()
    assert empty.summary()["shader_clock_mhz"] is None and empty.summary()["socket_power_w"] is None
