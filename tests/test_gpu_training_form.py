"""Training-form attention of the register-focused layers (Section 3.2, Training: for layer l > k only register and
generated tokens participate).  The teacher-forced sequence is [prefix registers; prompt; suffix registers; target tokens
Y]; the participating tokens of layers l > k are [prefix; suffix; Y] in original order at their original positions.  The
target tokens follow the suffix registers, so earn_compact_registers with t' = t + |Y| gathers exactly those rows, and
earn_prefill_attn on them with the gathered positions is the layer's forward.  Checked against the oracle's FULL-LENGTH
attention under the explicit key mask (key j allowed iff j is a register or target token and j <= i), read at those rows.
"""
import numpy as np
import pytest
import torch

from oracle import earn_oracle as O
from paper_2507_00715_amd import workloads as W
from parity import check_attn

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _B():
    from paper_2507_00715_amd import binding
    binding.lib()
    return binding


def masked_full_length_attention(q, k, v, cu, keep, hq, hkv, d):
    """Oracle-side definition: rotate at original positions (oracle_rope), then dense softmax under the key mask.
    Written with NumPy on the oracle's rotated tensors; evaluated only at the kept rows."""
    gq = hq // hkv
    out = {}
    for s in range(len(cu) - 1):
        sl = slice(cu[s], cu[s + 1])
        n = cu[s + 1] - cu[s]
        pos = np.arange(n)
        qr, kr = O.rope(q[sl], pos), O.rope(k[sl], pos)
        rows = np.nonzero(keep[sl])[0]
        o = np.zeros((len(rows), hq, d))
        for a in range(hq):
            sc = qr[rows, a] @ kr[:, a // gq].T / np.sqrt(d)
            allowed = keep[sl][None, :] & (pos[None, :] <= rows[:, None])
            sc = np.where(allowed, sc, -np.inf)
            p = np.exp(sc - sc.max(axis=1, keepdims=True))
            o[:, a] = (p / p.sum(axis=1, keepdims=True)) @ v[sl][:, a // gq]
        out[s] = o
    return out


@pytest.mark.parametrize("dtype,hq,hkv,d,h,t,y,prompts", [(torch.bfloat16, 8, 2, 128, 2, 2, 4, [300, 17, 1000]),
                                                           (torch.bfloat16, 14, 2, 64, 1, 1, 4, [64, 511]),
                                                           (torch.float32, 4, 4, 64, 2, 2, 3, [96, 128])])
def test_training_form_forward_of_register_layers(dtype, hq, hkv, d, h, t, y, prompts):
    B = _B()
    lens = [h + L + t + y for L in prompts]
    T, batch = sum(lens), len(lens)
    g = torch.Generator().manual_seed(T + y)
    rnd = lambda *s: torch.randn(*s, generator=g).to(dtype)
    q, k, v = rnd(T, hq, d), rnd(T, hkv, d), rnd(T, hkv, d)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    dcu = torch.from_numpy(cu).to(DEV)
    r = h + t + y
    dst = [torch.empty(batch * r, hh, d, dtype=dtype, device=DEV) for hh in (hq, hkv, hkv)]
    idx, pos = (torch.empty(batch * r, dtype=torch.int32, device=DEV) for _ in range(2))
    cu_c = torch.empty(batch + 1, dtype=torch.int32, device=DEV)
    B.earn_compact_registers([q.to(DEV), k.to(DEV), v.to(DEV)], dst, dcu, batch, h, t + y, idx, pos, cu_c)
    out = torch.full((batch * r, hq, d), float("nan"), dtype=dtype, device=DEV)
    desc = B.make_desc(dtype, hq, hkv, d)
    B.earn_prefill_attn(desc, dst[0], dst[1], dst[2], cu_c, pos, batch, batch * r, r, out, torch.empty_like(dst[1]), None, None)
    torch.cuda.synchronize()
    keep = np.zeros(T, dtype=bool)
    for s in range(batch):
        keep[cu[s]:cu[s] + h] = True
        keep[cu[s + 1] - t - y:cu[s + 1]] = True
    np.testing.assert_array_equal(idx.cpu().numpy(), np.nonzero(keep)[0])
    ref = masked_full_length_attention(W.to_f64(q), W.to_f64(k), W.to_f64(v), cu, keep, hq, hkv, d)
    for s in range(batch):
        check_attn(out[s * r:(s + 1) * r], ref[s], dtype, f"sequence {s}")
