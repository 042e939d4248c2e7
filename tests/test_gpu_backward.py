"""earn_attn_backward against the fp64 oracle (which is pinned against autograd of the library attention).

The HIP backward is fed what a training step has: rotated q and k, v, and the HIP FORWARD's out and lse (bf16 rounding of
`out` included), plus dOut.  The oracle differentiates the exact fp64 attention of the same q, k, v.
Bars: fp32 max-abs <= 1e-4 x max(1, max|ref|); bf16: tensor-wide relative Frobenius error <= 2e-2, per (row, head) vector
<= 2e-2 of the LARGEST vector norm of the tensor (gradient rows differ in scale by orders of magnitude: a late query's dq
is a difference of near-equal terms, so a vector is measured against the tensor's scale, not its own)."""
import numpy as np
import pytest
import torch

from oracle import earn_oracle as O
from paper_2507_00715_amd import workloads as W
from parity import rel_fro, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
BF, F32 = torch.bfloat16, torch.float32


def _B():
    from paper_2507_00715_amd import binding
    binding.lib()
    return binding


def check_grad(got, ref, dtype, what):
    g, r = to_np(got), to_np(ref)
    assert np.isfinite(g).all(), f"{what}: non-finite"
    if dtype == F32:
        err = np.abs(g - r).max()
        assert err <= 1e-4 * max(1.0, np.abs(r).max()), f"{what}: max-abs {err:.3e}"
        return
    assert rel_fro(g, r) <= 2e-2, f"{what}: rel-Frobenius {rel_fro(g, r):.3e}"
    vec = np.linalg.norm(g - r, axis=-1)
    assert vec.max() <= 2e-2 * np.linalg.norm(r, axis=-1).max(), f"{what}: worst vector off by {vec.max():.3e} (largest norm {np.linalg.norm(r, axis=-1).max():.3e})"


CASES = [
    # dtype, hq, hkv, d, lengths, softmax scale (0 = default)
    (F32, 4, 4, 64, [100, 132], 0.0),
    (F32, 6, 2, 128, [1, 63, 64, 65], 0.2),
    (BF, 14, 2, 64, [1, 59, 64, 300, 521], 0.0),
    (BF, 8, 2, 128, [700, 60, 129], 0.0),
    (BF, 4, 4, 128, [16] * 5, 0.0),            # register-focused layers: compacted sequences
]


@pytest.mark.parametrize("dtype,hq,hkv,d,lens,scale", CASES)
def test_attention_backward_matches_oracle(dtype, hq, hkv, d, lens, scale):
    B = _B()
    T, batch = sum(lens), len(lens)
    g = torch.Generator().manual_seed(T + hq)
    rnd = lambda *s: torch.randn(*s, generator=g).to(dtype)
    q, k, v, go = rnd(T, hq, d), rnd(T, hkv, d), rnd(T, hkv, d), rnd(T, hq, d)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    dcu = torch.from_numpy(cu).to(DEV)
    desc = B.make_desc(dtype, hq, hkv, d, scale, 0.0)      # rotation off: q, k are what the attention sees
    dq_, dk_, dv_, dgo = q.to(DEV), k.to(DEV), v.to(DEV), go.to(DEV)
    out = torch.empty(T, hq, d, dtype=dtype, device=DEV)
    lse = torch.empty(T, hq, dtype=torch.float32, device=DEV)
    B.earn_prefill_attn(desc, dq_, dk_, dv_, dcu, None, batch, T, max(lens), out, None, lse, None)
    gq, gk, gv = (torch.full(t.shape, float("nan"), dtype=dtype, device=DEV) for t in (q, k, v))
    B.earn_attn_backward(desc, dq_, dk_, dv_, out, lse, dgo, dcu, batch, T, max(lens), gq, gk, gv)
    torch.cuda.synchronize()
    ref = O.attn_backward(W.to_f64(q), W.to_f64(k), W.to_f64(v), W.to_f64(go), cu, scale=scale)
    check_grad(gq, ref["dq"], dtype, "dq")
    check_grad(gk, ref["dk"], dtype, "dk")
    check_grad(gv, ref["dv"], dtype, "dv")


def test_attention_backward_argument_errors():
    B = _B()
    z = torch.zeros(8, 2, 64, dtype=BF, device=DEV)
    lse = torch.zeros(8, 2, device=DEV)
    cu = torch.tensor([0, 8], dtype=torch.int32, device=DEV)
    with pytest.raises(B.EarnError) as e:
        B.earn_attn_backward(B.make_desc(BF, 2, 2, 64), z, z, z, z, lse, z, cu, 1, 8, 8, z.clone(), z.clone(), z.clone())
    assert e.value.code == B.EARN_ERR_UNSUPPORTED and "rope_base" in str(e.value)
    desc = B.make_desc(BF, 2, 2, 64, rope_base=0.0)
    with pytest.raises(B.EarnError) as e:
        B.earn_attn_backward(desc, z, z, z, z, None, z, cu, 1, 8, 8, z.clone(), z.clone(), z.clone())
    assert e.value.code == B.EARN_ERR_INVALID_ARG
    with pytest.raises(B.EarnError) as e:
        B.earn_attn_backward(desc, z, z, z, z, lse, z, cu, 1, 8, 8, z.clone(), z.clone(), z.clone(),
                             workspace=torch.empty(16, dtype=torch.uint8, device=DEV))
    assert e.value.code == B.EARN_ERR_WORKSPACE_TOO_SMALL
