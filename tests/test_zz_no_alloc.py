"""earn_decode_attn_static — the decode entry point for callers that cannot allocate — against earn_decode_attn on the
same inputs (same kernels, so bit for bit) and against the fp64 oracle, on two calls in a row, the second with a
smaller problem: the library's buffer keeps the first call's partial results, which must not leak into the second.
"""
import numpy as np
import pytest
import torch

from oracle import earn_oracle as O
from paper_2507_00715_amd import workloads as W
from parity import check_attn

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
BF, F32 = torch.bfloat16, torch.float32


def _B():
    from paper_2507_00715_amd import binding
    binding.lib()
    return binding


def one_call(B, dtype, hq, hkv, d, slens, beams, gen_cap, seed):
    batch, S = len(slens), len(slens) * beams
    g = torch.Generator().manual_seed(seed)
    rnd = lambda *s: torch.randn(*s, generator=g).to(dtype)
    cu = np.concatenate([[0], np.cumsum(slens)]).astype(np.int32)
    s2s = [u // beams for u in range(S)]
    glens = [(3 * u) % gen_cap for u in range(S)]
    sk, sv = rnd(int(cu[-1]), hkv, d), rnd(int(cu[-1]), hkv, d)
    q, kn, vn = rnd(S, hq, d), rnd(S, hkv, d), rnd(S, hkv, d)
    gk, gv = rnd(S, gen_cap, hkv, d), rnd(S, gen_cap, hkv, d)
    q_pos = [slens[s2s[u]] + glens[u] for u in range(S)]
    desc = B.make_desc(dtype, hq, hkv, d)
    need = B.earn_decode_workspace_bytes(desc, S, batch, max(slens), gen_cap)
    assert 0 < need <= B.EARN_STATIC_SCRATCH_BYTES, "the case must use scratch memory"
    dev = lambda x: x.to(DEV)
    i32 = lambda x: torch.tensor(list(x), dtype=torch.int32, device=DEV)
    args = (dev(q), dev(kn), dev(vn), i32(q_pos), dev(sk), dev(sv), i32(cu), i32(s2s))
    tail = (i32(glens), gen_cap, S, batch, max(slens))
    # the entry point under test
    gk_s, gv_s = dev(gk), dev(gv)
    out_s = torch.full((S, hq, d), float("nan"), dtype=dtype, device=DEV)
    B.earn_decode_attn_static(desc, *args, gk_s, gv_s, *tail, out_s)
    torch.cuda.synchronize()
    # the existing entry point, with a caller-owned workspace
    gk_w, gv_w = dev(gk), dev(gv)
    out_w = torch.full((S, hq, d), float("nan"), dtype=dtype, device=DEV)
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    B.earn_decode_attn(desc, *args, gk_w, gv_w, *tail, out_w, ws)
    torch.cuda.synchronize()
    assert torch.isfinite(out_s.float()).all()
    assert torch.equal(out_s, out_w) and torch.equal(gk_s, gk_w) and torch.equal(gv_s, gv_w)
    o_gk, o_gv = W.to_f64(gk), W.to_f64(gv)
    ref = O.decode_attn(W.to_f64(q), W.to_f64(kn), W.to_f64(vn), q_pos, W.to_f64(sk), W.to_f64(sv), cu, s2s, o_gk, o_gv,
                        glens)
    check_attn(out_s, ref["out"], dtype, "earn_decode_attn_static vs oracle")
    for u in range(S):
        check_attn(gk_s[u, glens[u]], o_gk[u, glens[u]], dtype, "appended key")


CASES = [
    # first call, then a smaller one: (dtype, hq, hkv, d, shared lengths, beams, gen_cap)
    ((BF, 8, 2, 128, [900, 129, 2000], 3, 4), (BF, 8, 2, 128, [300], 2, 4)),          # matrix-core kernel + combine
    ((BF, 32, 32, 128, [2059, 700], 1, 3), (BF, 32, 32, 128, [600], 1, 3)),           # vector kernel + combine
    ((F32, 4, 2, 64, [3000, 500], 2, 2), (BF, 14, 2, 64, [400, 130], 1, 2)),          # fp32, then another dtype and shape
]


@pytest.mark.parametrize("first,second", CASES)
def test_static_scratch_decode_two_calls_in_a_row(first, second):
    B = _B()
    one_call(B, *first, seed=1)
    one_call(B, *second, seed=2)


def test_static_scratch_decode_rejects_what_does_not_fit():
    B = _B()
    hq, hkv, d, batch, beams, gen_cap, n = 32, 8, 128, 16, 10, 8, 8256
    S = batch * beams
    desc = B.make_desc(BF, hq, hkv, d)
    B.earn_set_tuning("decode_mfma_wgs", 2048)      # many key splits: more partial results than the buffer holds
    try:
        assert B.earn_decode_workspace_bytes(desc, S, batch, n, gen_cap) > B.EARN_STATIC_SCRATCH_BYTES
        z = lambda *s: torch.zeros(*s, dtype=BF, device=DEV)
        i32 = lambda x: torch.tensor(list(x), dtype=torch.int32, device=DEV)
        out = torch.full((S, hq, d), 7.0, dtype=BF, device=DEV)
        sk = z(batch * n, hkv, d)
        with pytest.raises(B.EarnError) as e:
            B.earn_decode_attn_static(desc, z(S, hq, d), z(S, hkv, d), z(S, hkv, d), i32([n] * S), sk, sk,
                                      i32(range(0, batch * n + 1, n)), i32([u // beams for u in range(S)]),
                                      z(S, gen_cap, hkv, d), z(S, gen_cap, hkv, d), i32([0] * S), gen_cap, S, batch, n, out)
        assert e.value.code == B.EARN_ERR_WORKSPACE_TOO_SMALL and "use earn_decode_attn" in str(e.value)
        torch.cuda.synchronize()
        assert (out == 7.0).all()
    finally:
        B.earn_set_tuning("decode_mfma_wgs", 0)
