"""The seeded input generator: determinism, restriction invariance, distribution, layout."""
import numpy as np
import torch

from paper_2507_00715_amd import workloads as W


def test_values_match_the_python_int_reference():
    w = W.Workload(W.CONFIGS["small_gqa"])
    q = w.prefill_tensor("q", 3, seqs=[5])
    key = w._key(3, W.T_Q)
    table = W.normal_table()
    for pos, head, e in [(0, 0, 0), (17, 5, 9), (200, 13, 63)]:
        z = key ^ ((5 << 40) | (pos << 20) | (head * 64 + e))
        want = table[W.mix64_int(z) >> 48].to(torch.bfloat16)
        assert q[pos, head, e] == want


def test_restriction_invariance_and_determinism():
    w = W.Workload(W.CONFIGS["tiny_f32"])
    k = w.prefill_tensor("k", 1)
    assert k.shape == (232, 4, 64) and k.dtype == torch.float32
    assert torch.equal(k, W.Workload(W.CONFIGS["tiny_f32"]).prefill_tensor("k", 1))
    s0, s1 = w.cu_seqlens[1], w.cu_seqlens[2]
    assert torch.equal(w.prefill_tensor("k", 1, seqs=[1], heads=[3, 0]), k[s0:s1][:, [3, 0]])
    assert not torch.equal(k, w.prefill_tensor("k", 2))
    assert not torch.equal(k, w.prefill_tensor("v", 1))


def test_layout_matches_the_configurations():
    w = W.Workload(W.CONFIGS["tiny_f32"])
    assert w.seq_lengths == [100, 132] and w.total_tokens == 232 and w.causal_pairs() == 13828
    w2 = W.Workload(W.CONFIGS["small_gqa"])
    assert all(256 <= L <= 512 for L in w2.history_lengths) and len(set(w2.history_lengths)) > 16
    w4 = W.Workload(W.CONFIGS["long_beam"])
    assert w4.total_tokens == 16 * 8256 and w4.n_streams == 160 and w4.stream_to_seq[19] == 1
    w5 = W.Workload(W.CONFIGS["serving"])
    assert all(64 <= L <= 1024 for L in w5.history_lengths)
    assert np.median(w5.history_lengths) < 400          # log-uniform: the median sits near sqrt(64*1024) = 256
    assert w4.decode_positions(2)[0] == 8258


def test_distribution_and_outliers():
    w = W.Workload(W.CONFIGS["mid_mha"])
    seq = torch.zeros(600, dtype=torch.int64)
    pos = torch.arange(600)
    v = w.prefill_tensor("v", 0, coords=(seq, pos)).float()
    assert abs(v.mean()) < 5e-3 and abs(v.std() - 1) < 5e-3
    k = w.prefill_tensor("k", 0, coords=(seq, pos)).float()
    frac = (k.std(dim=-1) > 4).float().mean().item()      # rows scaled x8 have std ~ 8
    assert 0.035 < frac < 0.065


def test_decode_tensors():
    w = W.Workload(W.CONFIGS["long_beam"])
    q = w.decode_tensor("q", 7, 3, streams=[0, 1, 159])
    assert q.shape == (3, 32, 128)
    assert torch.equal(q[1:2], w.decode_tensor("q", 7, 3, streams=[1]))
    assert not torch.equal(q[0], q[1])
