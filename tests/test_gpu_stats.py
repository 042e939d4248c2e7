"""earn_attn_stats (Sparsity / Sink_head / Sink_tail of chosen query rows) against the fp64 oracle.

Sink sums are floating point: within 1e-2 (bf16 operands) or 1e-4 (fp32) of the oracle.  Sparsity is a COUNT decided by a
floating-point comparison p > epsilon; a probability that sits within rounding of epsilon may fall either way, so the
count is checked to lie between the oracle's counts at epsilon (1 + delta) and epsilon (1 - delta), delta = the relative
accuracy of a probability in the kernel's arithmetic (3e-2 for bf16 operands, 1e-4 for fp32), and to EQUAL the oracle's
count wherever those two agree.
"""
import numpy as np
import pytest
import torch

from oracle import earn_oracle as O
from paper_2507_00715_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
BF, F32 = torch.bfloat16, torch.float32


def _B():
    from paper_2507_00715_amd import binding
    binding.lib()
    return binding


CASES = [
    # dtype, hq, hkv, d, h, t, sequence lengths, query scale (larger = more peaked rows)
    (BF, 8, 2, 128, 4, 4, [300, 64, 1000, 9], 1.0),
    (BF, 14, 2, 64, 2, 6, [17, 530, 2100], 3.0),
    (BF, 4, 4, 64, 0, 1, [50, 700, 1], 2.0),            # the last row only
    (F32, 6, 2, 128, 3, 3, [81, 300, 7], 2.0),
    (F32, 4, 4, 64, 2, 2, [100, 132], 1.0),
]


@pytest.mark.parametrize("dtype,hq,hkv,d,h,t,lens,qscale", CASES)
def test_attention_statistics_match_oracle(dtype, hq, hkv, d, h, t, lens, qscale):
    B = _B()
    r, batch, T = h + t, len(lens), sum(lens)
    g = torch.Generator().manual_seed(T + hq)
    rnd = lambda *s: torch.randn(*s, generator=g).to(dtype)
    q, k, v = (rnd(T, hq, d) * qscale).to(dtype), rnd(T, hkv, d), rnd(T, hkv, d)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    comp = O.compact_registers(None, cu, h, t)
    desc = B.make_desc(dtype, hq, hkv, d)
    dcu = torch.from_numpy(cu).to(DEV)
    # the layer's cache (rotated keys) from the prefill entry point, as in the path
    krot = torch.empty(T, hkv, d, dtype=dtype, device=DEV)
    B.earn_prefill_attn(desc, q.to(DEV), k.to(DEV), v.to(DEV), dcu, None, batch, T, max(lens),
                        torch.empty(T, hq, d, dtype=dtype, device=DEV), krot, None, None)
    q_rows = q[torch.from_numpy(comp["idx"]).long()].contiguous().to(DEV)
    stats = torch.full((batch * r, hq, 3), float("nan"), dtype=torch.float32, device=DEV)
    B.earn_attn_stats(desc, q_rows, krot, dcu, torch.from_numpy(comp["pos"]).to(DEV), batch, r, stats)
    torch.cuda.synchronize()
    got = stats.cpu().double().numpy()
    assert np.isfinite(got).all()
    sel = np.zeros(T, dtype=np.uint8)
    sel[comp["idx"]] = 1
    delta, atol = (3e-2, 1e-2) if dtype == BF else (1e-4, 1e-4)
    f64 = lambda x: W.to_f64(x)
    ref = O.attn_stats(f64(q), f64(k), cu, row_sel=sel)[comp["idx"]]
    lo = O.attn_stats(f64(q), f64(k), cu, row_sel=sel, epsilon=0.05 * (1 + delta))[comp["idx"]]
    hi = O.attn_stats(f64(q), f64(k), cu, row_sel=sel, epsilon=0.05 * (1 - delta))[comp["idx"]]
    n_keys = (comp["pos"] + 1)[:, None].astype(np.float64)
    cnt = lambda x: np.rint(x[:, :, 0] * n_keys)
    got_cnt = got[:, :, 0] * n_keys
    assert np.abs(got_cnt - np.rint(got_cnt)).max() < 1e-3             # it is a count
    got_cnt = np.rint(got_cnt)
    assert (cnt(lo) <= got_cnt).all() and (got_cnt <= cnt(hi)).all()
    sure = cnt(lo) == cnt(hi)
    assert sure.mean() > 0.8 and (got_cnt[sure] == cnt(ref)[sure]).all()
    assert cnt(ref).max() >= 2                                          # the case is not trivially empty
    assert np.abs(got[:, :, 1:] - ref[:, :, 1:]).max() <= atol, np.abs(got[:, :, 1:] - ref[:, :, 1:]).max()


def test_attention_statistics_argument_errors():
    B = _B()
    desc = B.make_desc(BF, 4, 2, 64)
    z = torch.zeros(8, 4, 64, dtype=BF, device=DEV)
    kz = torch.zeros(8, 2, 64, dtype=BF, device=DEV)
    cu = torch.tensor([0, 8], dtype=torch.int32, device=DEV)
    pos = torch.tensor([7], dtype=torch.int32, device=DEV)
    out = torch.zeros(1, 4, 3, device=DEV)
    with pytest.raises(B.EarnError):
        B.earn_attn_stats(desc, z, kz, cu, pos, 1, 0, out)
    with pytest.raises(B.EarnError):
        B.earn_attn_stats(desc, z, kz, cu, pos, 1, 1, out, epsilon=-1.0)
    with pytest.raises(B.EarnError):
        B.earn_attn_stats(desc, None, kz, cu, pos, 1, 1, out)
    B.earn_attn_stats(desc, z[7:8].contiguous(), kz, cu, pos, 1, 1, out)   # uniform row of 8 keys
    torch.cuda.synchronize()
    np.testing.assert_allclose(out.cpu().numpy()[0], [[1.0, 3 / 8, 4 / 8]] * 4, rtol=1e-6)
