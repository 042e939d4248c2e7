"""Host-side parts of bench.py (no GPU): the algorithmic work counts behind the reported rates, pinned to the closed
forms and to the figures of the configurations; and the command line's refusal of more than one GPU."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402
from paper_2507_00715_amd import workloads as W  # noqa: E402


def test_prefill_flops_are_the_causal_pair_count():
    # fixed-length configuration: closed form 4 d Hq B n (n + 1) / 2 (QK^T and PV, 2 d each per allowed pair)
    w = W.Workload(W.CONFIGS["long_beam"])
    c = w.cfg
    n = c.n_head_reg + 8192 + c.n_tail_reg
    assert w.seq_lengths == [n] * c.batch
    alg = bench.algorithmic_counts(w)
    assert alg["flops_full"] == 4.0 * c.head_dim * c.n_q_heads * c.batch * n * (n + 1) / 2
    assert abs(alg["flops_full"] / 8.94e12 - 1) < 2e-3          # the configuration's quoted 8.94 TFLOP per layer
    r = c.r
    assert alg["flops_reg"] == 4.0 * c.head_dim * c.n_q_heads * c.batch * r * (r + 1) / 2
    # ragged configuration: brute force over the drawn lengths
    w = W.Workload(W.CONFIGS["small_gqa"])
    c = w.cfg
    pairs = sum(i + 1 for n in w.seq_lengths for i in range(n))
    assert bench.algorithmic_counts(w)["flops_full"] == 4.0 * c.head_dim * c.n_q_heads * pairs


def test_executed_tile_flops_bound_the_algorithmic_ones():
    for name in ("small_gqa", "mid_mha", "long_beam", "serving"):
        w = W.Workload(W.CONFIGS[name])
        alg, exe = bench.algorithmic_counts(w)["flops_full"], bench.executed_tile_flops(w)
        assert alg < exe < 1.35 * alg
    # one sequence of 64 rows: two waves, each multiplies the one 64-key tile: 2 * 32 * 64 pairs
    cfg = W.CONFIGS["small_gqa"].replace(batch=1, n_head_reg=0, n_tail_reg=1)
    w = W.Workload(cfg, history_lengths=[63])
    assert bench.executed_tile_flops(w) == 4.0 * cfg.head_dim * cfg.n_q_heads * 2 * 32 * 64


def test_decode_and_compaction_bytes():
    w = W.Workload(W.CONFIGS["long_beam"])
    c = w.cfg
    alg = bench.algorithmic_counts(w)
    e, S = 2, c.batch * c.beams
    row = c.n_kv_heads * c.head_dim * e
    # full-cache layer, step g: shared rows once per SEQUENCE, g+1 generated rows per stream, q/o, k_new/v_new in + out
    for g in (0, c.decode_steps - 1):
        want = 2 * row * (w.total_tokens + S * (g + 1)) + 2 * c.n_q_heads * c.head_dim * e * S + 4 * row * S
        assert alg["dec_full"][g] == want
    assert abs(alg["dec_full"][0] / 0.54e9 - 1) < 0.03           # the configuration's quoted 0.54 GB per layer and step
    want_reg = 2 * row * (c.batch * c.r + S) + 2 * c.n_q_heads * c.head_dim * e * S + 4 * row * S
    assert alg["dec_reg"][0] == want_reg
    # compaction: hidden-state stand-in + Q, K, V of the N-k later layers, read and written, plus the index outputs
    rows = c.batch * c.r
    per_layer = (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim * e
    want = 2 * rows * (c.n_q_heads * c.head_dim * e + (c.n_layers - c.split_k) * per_layer) + 12 * rows + 8 * c.batch
    assert alg["compaction"] == want


def test_prefill_bytes_per_layer():
    c = W.CONFIGS["long_beam"]
    T = c.batch * (c.n_head_reg + 8192 + c.n_tail_reg)
    # Q in, O out (Hq rows each); K in, rotated K out, V in (Hkv rows each)
    assert bench.algorithmic_prefill_bytes("long_beam") == T * c.head_dim * 2 * (2 * c.n_q_heads + 3 * c.n_kv_heads)


@pytest.mark.parametrize("args", [["--gpus", "2"], ["--gpus", "8"]])
def test_more_than_one_gpu_is_refused(args):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "single-GPU" in r.stderr and r.stdout.strip() == ""
