"""Parity of both full-length bf16 prefill kernels (256-row workgroups, software pipelined; 128-row workgroups, plain
schedule) on a RAGGED batch with sequences of more than 4000 rows: the others end inside a workgroup, inside a wave's
32 rows, inside a 64-key tile, or are shorter than one tile.  (By itself earn_prefill_attn gives such a batch, short
on average, to the 128-row form; the tuning key selects either.)  A few key rows are scaled up (outliers), so the
running softmax reference jumps and the exact-recompute path of the kernels runs too.

Attention outputs are checked against the fp64 oracle on sampled rows (every row of the short sequences); inputs are
drawn on the GPU and again on the CPU from the same counter-based generator.
"""
import numpy as np
import pytest
import torch

from oracle import earn_oracle as O
from paper_2507_00715_amd import workloads as W
from parity import BF16_REL, check_attn, rel_fro, vector_bar

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
# n_s = r + L_s with r = 16: 17, 64, 65, 300, 3100, 4100 tokens
HISTORY = (1, 48, 49, 284, 3084, 4084)


def _B():
    from paper_2507_00715_amd import binding
    binding.lib()
    return binding


# outlier keys 8 times the usual scale move the row maxima by a few binary orders (the stale reference absorbs that);
# 24 times moves them by dozens: the kernel has to re-reference in the middle of a sequence (exact path)
@pytest.mark.parametrize("block_rows", [256, 128])
@pytest.mark.parametrize("head_dim,outlier_scale", [(128, 8.0), (64, 8.0), (128, 24.0), (64, 24.0)])
def test_pipelined_prefill_ragged_batch_with_outliers(head_dim, outlier_scale, block_rows):
    B = _B()
    B.earn_set_tuning("prefill_block_rows", block_rows)
    try:
        _ragged_batch_with_outliers(B, head_dim, outlier_scale)
    finally:
        B.earn_set_tuning("prefill_block_rows", 0)


def _ragged_batch_with_outliers(B, head_dim, outlier_scale):
    cfg = W.CONFIGS["mid_mha"].replace(name="ragged_long", config_id=41, batch=len(HISTORY), len_dist=("list", HISTORY),
                                       n_head_reg=8, n_tail_reg=8, n_q_heads=4, n_kv_heads=2, head_dim=head_dim,
                                       outlier_prob=0.05, outlier_scale=outlier_scale)
    w = W.Workload(cfg)
    assert w.max_seqlen > 3072
    coords = w.token_coords(DEV)
    q, k, v = (w.prefill_tensor(t, 0, coords=coords) for t in "qkv")
    out = torch.full_like(q, float("nan"))
    krot = torch.empty_like(k)
    lse = torch.empty(w.total_tokens, cfg.n_q_heads, dtype=torch.float32, device=DEV)
    cu = torch.tensor(w.cu_seqlens, dtype=torch.int32, device=DEV)
    desc = B.make_desc(cfg.torch_dtype, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, 0.0, cfg.rope_base)
    B.earn_prefill_attn(desc, q, k, v, cu, None, cfg.batch, w.total_tokens, w.max_seqlen, out, krot, lse, None)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()

    rng = np.random.default_rng(7)
    gq = cfg.n_q_heads // cfg.n_kv_heads
    heads = list(range(cfg.n_q_heads))
    for s, n in enumerate(w.seq_lengths):
        b0 = w.cu_seqlens[s]
        qc = W.to_f64(w.prefill_tensor("q", 0, seqs=[s]))
        kc = W.to_f64(w.prefill_tensor("k", 0, seqs=[s]))
        vc = W.to_f64(w.prefill_tensor("v", 0, seqs=[s]))
        if n <= 300:
            rows = list(range(n))
        else:  # rows around wave (32), tile (64) and workgroup (256) boundaries, the ends, and random rows
            rows = set(range(16)) | set(range(n - 16, n))
            for b in (32, 64, 256):
                for edge in range(b, n, b * 5):
                    rows.update(r for r in (edge - 1, edge, edge + 1) if r < n)
            rows.update(int(x) for x in rng.integers(0, n, size=48))
            rows = sorted(rows)
        sel = np.zeros(n, dtype=np.uint8)
        sel[rows] = 1
        ref = O.prefill_attn(qc, kc, vc, [0, n], q_to_kv=[a // gq for a in heads], rope_base=cfg.rope_base, row_sel=sel)
        got = out[b0:b0 + n][rows].cpu().double().numpy()
        # per (row, head) vector as well: a wrong tile shows in single rows long before it moves the norm of the sample
        check_attn(got, ref["out"][rows], torch.bfloat16, f"d={head_dim} seq {s} (n={n}), {len(rows)} rows",
                   vector_bar(outlier_scale))
        got_lse = lse[b0:b0 + n][rows].cpu().double().numpy()
        assert (np.abs(got_lse - ref["lse"][rows]) <= 5e-2 + 1e-2 * np.abs(ref["lse"][rows])).all()
        check_attn(krot[b0:b0 + n], ref["k_rot"], torch.bfloat16, f"d={head_dim} seq {s} rotated keys")
