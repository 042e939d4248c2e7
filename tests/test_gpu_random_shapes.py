"""Seeded sweep over randomly drawn (valid) shapes: head counts and group sizes, both head dimensions, ragged caches
including empty ones, uneven beam counts (sequences without any stream included), ragged generated lengths, and
register counts.  Every case is checked against the fp64 oracle to the usual bars; the point is the shapes nobody
thought of when writing the targeted cases, so the draws are fixed by the seed and the case number names them.
"""
import numpy as np
import pytest
import torch

from oracle import earn_oracle as O
from paper_2507_00715_amd import workloads as W

from parity import check_attn as check

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _B():
    from paper_2507_00715_amd import binding
    binding.lib()
    return binding


def draw_heads(rng):
    hkv = int(rng.choice([1, 2, 3, 4, 8]))
    gq = int(rng.choice([1, 1, 2, 3, 4, 5, 6, 7, 8]))
    return hkv * gq, hkv, int(rng.choice([64, 128]))


@pytest.mark.parametrize("case", range(24))
def test_decode_random_shape(case):
    B = _B()
    rng = np.random.default_rng(7000 + case)
    dtype = torch.float32 if case % 6 == 5 else torch.bfloat16
    hq, hkv, d = draw_heads(rng)
    batch = int(rng.integers(1, 6))
    slens = [int(x) for x in rng.choice([0, 1, 15, 64, 65, 127, 128, 129, 300, 700], size=batch)]
    beams_of = [int(x) for x in rng.choice([0, 1, 1, 2, 3, 9, 21], size=batch)]
    if sum(beams_of) == 0:
        beams_of[0] = 1
    s2s = [s for s in range(batch) for _ in range(beams_of[s])]
    S = len(s2s)
    gen_cap = int(rng.choice([1, 2, 5, 70]))
    glens = [int(x) for x in rng.integers(0, gen_cap, size=S)]
    gtor = torch.Generator().manual_seed(case)
    rnd = lambda *shape: torch.randn(*shape, generator=gtor).to(dtype)
    cu = np.concatenate([[0], np.cumsum(slens)]).astype(np.int32)
    T = int(cu[-1])
    sk, sv = rnd(max(T, 1), hkv, d)[:T], rnd(max(T, 1), hkv, d)[:T]
    q, kn, vn = rnd(S, hq, d), rnd(S, hkv, d), rnd(S, hkv, d)
    gk, gv = rnd(S, gen_cap, hkv, d), rnd(S, gen_cap, hkv, d)
    q_pos = [slens[s2s[u]] + glens[u] for u in range(S)]
    desc = B.make_desc(dtype, hq, hkv, d)
    dev = lambda x: x.contiguous().to(DEV)
    i32 = lambda x: torch.tensor(list(x), dtype=torch.int32, device=DEV)
    d_sk = dev(sk) if T else torch.zeros(1, hkv, d, dtype=dtype, device=DEV)
    d_sv = dev(sv) if T else torch.zeros(1, hkv, d, dtype=dtype, device=DEV)
    d_gk, d_gv = dev(gk), dev(gv)
    out = torch.full((S, hq, d), float("nan"), dtype=dtype, device=DEV)
    ws = torch.empty(max(B.earn_decode_workspace_bytes(desc, S, batch, max(slens), gen_cap), 1), dtype=torch.uint8,
                     device=DEV)
    print(f"case {case}: {dtype} hq={hq} hkv={hkv} d={d} slens={slens} beams={beams_of} gen_cap={gen_cap}", flush=True)
    B.earn_decode_attn(desc, dev(q), dev(kn), dev(vn), i32(q_pos), d_sk, d_sv, i32(cu), i32(s2s), d_gk, d_gv,
                       i32(glens), gen_cap, S, batch, max(slens), out, ws)
    torch.cuda.synchronize()
    o_gk, o_gv = W.to_f64(gk), W.to_f64(gv)
    ref = O.decode_attn(W.to_f64(q), W.to_f64(kn), W.to_f64(vn), q_pos, W.to_f64(sk), W.to_f64(sv), cu, s2s, o_gk, o_gv,
                        glens)
    for u in range(S):
        check(out[u], ref["out"][u], dtype, f"case {case} stream {u}")
        check(d_gk[u, glens[u]], o_gk[u, glens[u]], dtype, f"case {case} appended key of stream {u}")
        assert torch.equal(d_gv[u, glens[u]].cpu(), vn[u])
        keep = [j for j in range(gen_cap) if j != glens[u]]
        assert torch.equal(d_gk[u, keep].cpu(), gk[u, keep]) and torch.equal(d_gv[u, keep].cpu(), gv[u, keep])


@pytest.mark.parametrize("case", range(16))
def test_prefill_and_register_rows_random_shape(case):
    B = _B()
    rng = np.random.default_rng(9000 + case)
    dtype = torch.float32 if case % 8 == 7 else torch.bfloat16
    hq, hkv, d = draw_heads(rng)
    h, t = int(rng.choice([0, 1, 2, 8, 17, 32])), int(rng.choice([0, 1, 3, 8, 16, 33]))
    if h + t == 0:
        t = 1
    r = h + t
    batch = int(rng.integers(1, 5))
    lens = [r + int(x) for x in rng.choice([0, 1, 30, 63, 64, 200, 500, 1100], size=batch)]
    T = sum(lens)
    gtor = torch.Generator().manual_seed(100 + case)
    rnd = lambda *shape: torch.randn(*shape, generator=gtor).to(dtype)
    q, k, v = rnd(T, hq, d), rnd(T, hkv, d), rnd(T, hkv, d)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    d_cu = torch.from_numpy(cu).to(DEV)
    d_q, d_k, d_v = q.to(DEV), k.to(DEV), v.to(DEV)
    desc = B.make_desc(dtype, hq, hkv, d)
    print(f"case {case}: {dtype} hq={hq} hkv={hkv} d={d} h={h} t={t} lens={lens}", flush=True)

    # the whole layer
    out = torch.full((T, hq, d), float("nan"), dtype=dtype, device=DEV)
    k_rot = torch.empty_like(d_k)
    B.earn_prefill_attn(desc, d_q, d_k, d_v, d_cu, None, batch, T, max(lens), out, k_rot, None, None)
    torch.cuda.synchronize()
    ref = O.prefill_attn(W.to_f64(q), W.to_f64(k), W.to_f64(v), cu)
    for s in range(batch):
        check(out[cu[s]:cu[s + 1]], ref["out"][cu[s]:cu[s + 1]], dtype, f"case {case} prefill sequence {s}")
    check(k_rot, ref["k_rot"], dtype, f"case {case} rotated keys")

    # its register rows only
    q_rows = torch.empty(batch * r, hq, d, dtype=dtype, device=DEV)
    idx, pos = (torch.empty(batch * r, dtype=torch.int32, device=DEV) for _ in range(2))
    cu_c = torch.empty(batch + 1, dtype=torch.int32, device=DEV)
    B.earn_compact_registers([d_q], [q_rows], d_cu, batch, h, t, idx, pos, cu_c)
    out_rows = torch.full((batch * r, hq, d), float("nan"), dtype=dtype, device=DEV)
    k_rot2 = torch.empty_like(d_k)
    ws = torch.empty(max(B.earn_prefill_register_rows_workspace_bytes(desc, batch, max(lens), r), 256),
                     dtype=torch.uint8, device=DEV)
    B.earn_prefill_register_rows(desc, q_rows, d_k, d_v, d_cu, pos, batch, T, max(lens), r, out_rows, k_rot2, ws)
    torch.cuda.synchronize()
    ref_c = O.compact_registers(None, cu, h, t)
    np.testing.assert_array_equal(idx.cpu().numpy(), ref_c["idx"])
    want = ref["out"][ref_c["idx"]]
    for s in range(batch):
        check(out_rows[s * r:(s + 1) * r], want[s * r:(s + 1) * r], dtype, f"case {case} register rows of sequence {s}")
    assert torch.equal(k_rot2, k_rot)


@pytest.mark.parametrize("case", range(8))
def test_compaction_random_shape(case):
    """Random register counts, ragged lengths (sequences that are all registers included), 1 to 112 tensors of random
    row widths in one launch: bit-exact against the oracle's gather of the same bytes."""
    B = _B()
    rng = np.random.default_rng(11000 + case)
    h, t = int(rng.choice([0, 1, 3, 8, 32])), int(rng.choice([0, 1, 2, 16, 32]))
    if h + t == 0:
        h = 1
    r = h + t
    batch = int(rng.integers(1, 40))
    lens = [r + int(x) for x in rng.choice([0, 0, 1, 5, 64, 333, 2000], size=batch)]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T = int(cu[-1])
    n_tensors = int(rng.choice([1, 2, 7, 40, 112]))
    widths = [int(x) for x in rng.choice([16, 32, 48, 256, 512, 4096, 8208], size=n_tensors)]   # row bytes
    if n_tensors > 7:   # keep the byte volume of the many-tensor cases small
        widths = [min(wd, 512) for wd in widths]
    print(f"case {case}: h={h} t={t} batch={batch} T={T} tensors={n_tensors} widths={sorted(set(widths))}", flush=True)
    g = torch.Generator().manual_seed(case)
    srcs = [torch.randint(0, 256, (T, wd), dtype=torch.uint8, generator=g) for wd in widths]
    d_src = [s.to(DEV) for s in srcs]
    d_dst = [torch.full((batch * r, wd), 0xEE, dtype=torch.uint8, device=DEV) for wd in widths]
    d_cu = torch.from_numpy(cu).to(DEV)
    idx, pos = (torch.full((batch * r,), -1, dtype=torch.int32, device=DEV) for _ in range(2))
    cu_c = torch.full((batch + 1,), -1, dtype=torch.int32, device=DEV)
    B.earn_compact_registers(d_src, d_dst, d_cu, batch, h, t, idx, pos, cu_c)
    torch.cuda.synchronize()
    ref = O.compact_registers(None, cu, h, t)
    np.testing.assert_array_equal(idx.cpu().numpy(), ref["idx"])
    np.testing.assert_array_equal(pos.cpu().numpy(), ref["pos"])
    np.testing.assert_array_equal(cu_c.cpu().numpy(), ref["cu"])
    for s, dd in zip(srcs, d_dst):
        assert np.array_equal(dd.cpu().numpy(), O.compact_registers(s.numpy(), cu, h, t)["dst"])
