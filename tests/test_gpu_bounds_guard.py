"""The kernels hold sequence bounds inside the row counts they are told (total_tokens / shared_total), whatever
cu_seqlens / shared_cu say.  Checked without any risk to the GPU: every tensor handed over is the first half of an
allocation twice as large, so even an unguarded kernel would stay inside allocated memory; the assertion is that a
bound reaching past the told row count gives exactly what the same call gives with that bound cut back to it."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
BF = torch.bfloat16


def _B():
    from paper_2507_00715_amd import binding
    binding.lib()
    return binding


def half(*shape, dtype=BF, seed=0):
    """First half (along rows) of a random tensor twice as long."""
    g = torch.Generator(device=DEV).manual_seed(seed)
    big = torch.randn(2 * shape[0], *shape[1:], device=DEV, generator=g).to(dtype)
    return big[:shape[0]]


def i32(a):
    return torch.tensor(list(a), dtype=torch.int32, device=DEV)


@pytest.mark.parametrize("dtype", [BF, torch.float32])
def test_prefill_bounds_past_total_tokens_are_cut_back(dtype):
    B = _B()
    hq, hkv, d, lens = 4, 2, 64, [70, 130, 200]
    T = sum(lens)
    q, k, v = half(T, hq, d, dtype=dtype, seed=1), half(T, hkv, d, dtype=dtype, seed=2), half(T, hkv, d, dtype=dtype, seed=3)
    desc = B.make_desc(dtype, hq, hkv, d)
    good = [0, 70, 200, T]
    outs = []
    for cu in (good, [0, 70, 200, T + 90]):          # the last sequence claims 90 rows more than the tensors are said to hold
        out, krot = torch.zeros(T, hq, d, dtype=dtype, device=DEV), torch.zeros(T, hkv, d, dtype=dtype, device=DEV)
        B.earn_prefill_attn(desc, q, k, v, i32(cu), None, len(lens), T, 300, out, krot)
        torch.cuda.synchronize()
        outs.append((out, krot))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
    assert torch.isfinite(outs[1][0].float()).all()


def test_decode_bounds_past_shared_total_are_cut_back():
    B = _B()
    hq, hkv, d, batch, G = 4, 2, 128, 3, 4
    lens = [40, 150, 90]
    T = sum(lens)
    sk, sv = half(T, hkv, d, seed=4), half(T, hkv, d, seed=5)
    g = torch.Generator(device=DEV).manual_seed(6)
    rnd = lambda *s: torch.randn(*s, device=DEV, generator=g).to(BF)
    for beams in (1, 3):                              # the vector kernel, the matrix-core kernel
        S = batch * beams
        q, kn, vn = rnd(S, hq, d), rnd(S, hkv, d), rnd(S, hkv, d)
        s2s = i32([u // beams for u in range(S)]) if beams > 1 else None
        desc = B.make_desc(BF, hq, hkv, d)
        ws = torch.empty(max(B.earn_decode_workspace_bytes(desc, S, batch, 200, G), 256), dtype=torch.uint8, device=DEV)
        outs = []
        for cu in ([0, 40, 190, T], [0, 40, 190, T + 60]):
            gk, gv = torch.zeros(S, G, hkv, d, dtype=BF, device=DEV), torch.zeros(S, G, hkv, d, dtype=BF, device=DEV)
            out = torch.zeros(S, hq, d, dtype=BF, device=DEV)
            B.earn_decode_attn(desc, q, kn, vn, i32([300] * S), sk, sv, i32(cu), s2s, gk, gv, i32([0] * S), G, S, batch, 200,
                               out, ws)
            torch.cuda.synchronize()
            outs.append(out)
        assert torch.equal(outs[0], outs[1]) and torch.isfinite(outs[1].float()).all()


def test_compaction_rows_past_total_tokens_are_cut_back():
    B = _B()
    lens, h, t = [30, 50], 4, 4
    T = sum(lens)
    x = half(T, 64, dtype=torch.float32, seed=7)
    outs = []
    for cu in ([0, 30, T], [0, 30, T + 25]):
        dst = torch.zeros(len(lens) * (h + t), 64, dtype=torch.float32, device=DEV)
        idx = torch.zeros(len(lens) * (h + t), dtype=torch.int32, device=DEV)
        B.earn_compact_registers([x], [dst], i32(cu), len(lens), h, t, idx)
        torch.cuda.synchronize()
        outs.append((dst, idx))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
    assert int(outs[1][1].max()) < T
