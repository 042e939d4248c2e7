"""earn_qkv_rope_project and earn_linear against the fp64 oracle, and the projection-fed attention path (rotation done by
the projection's epilogue, attention called with rotation off and keys read in place) against the oracle's attention on
the oracle's projections."""
import numpy as np
import pytest
import torch

from oracle import earn_oracle as O
from paper_2507_00715_amd import workloads as W
from parity import check_attn

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
BF = torch.bfloat16


def _B():
    from paper_2507_00715_amd import binding
    binding.lib()
    return binding


def rnd(g, *shape, scale=1.0):
    return (torch.randn(*shape, generator=g) * scale).to(BF)


def wt(w):
    """The library takes weights as [outputs, inputs]; the oracle's matrices here are [inputs, outputs]."""
    return w.t().contiguous().to(DEV)


QKV_CASES = [
    # hq, hkv, d, d_model, sequence lengths, explicit positions
    (8, 2, 128, 256, [300, 61, 100], False),        # 12 heads x 128 = 1536 columns, ragged last row tile
    (14, 2, 64, 896, [17, 530], False),             # d = 64: two heads per column tile; 18 heads = 1152 columns (9 tiles)
    (4, 4, 128, 64, [40], True),                    # one k-tile, explicit positions (compacted register rows)
    (6, 2, 64, 192, [5, 1, 250], True),
    (8, 2, 128, 2048, [40, 17], True),              # few rows, long inner dimension: split over workgroups when allowed
    (14, 2, 64, 1024, [33], False),
]


@pytest.fixture(params=[1, 2], ids=["tile256x128", "tile256x256"])
def tile(request):
    """Both tile shapes of the GEMM kernel, whatever the library would pick for the size."""
    B = _B()
    B.earn_set_tuning("linear_tile", request.param)
    yield request.param
    B.earn_set_tuning("linear_tile", 0)


@pytest.fixture(params=["auto", None, 3], ids=["split-if-few-rows", "no-workspace", "three-splits"])
def ws(request):
    """With a workspace a few-row product splits its inner dimension (partial sums + a second kernel); without, never.
    The third form forces three splits whatever the size (an inner dimension of fewer K-tiles takes one split per tile)."""
    if request.param == 3:
        B = _B()
        B.earn_set_tuning("linear_splits", 3)
        yield "auto"
        B.earn_set_tuning("linear_splits", 0)
    else:
        yield request.param


@pytest.mark.parametrize("hq,hkv,d,dm,lens,explicit", QKV_CASES)
def test_qkv_projection_matches_oracle(hq, hkv, d, dm, lens, explicit, tile, ws):
    B = _B()
    rows, batch = sum(lens), len(lens)
    g = torch.Generator().manual_seed(rows + dm)
    x, w = rnd(g, rows, dm), rnd(g, dm, (hq + 2 * hkv) * d, scale=dm ** -0.5)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    pos = np.concatenate([np.arange(n) for n in lens]).astype(np.int32)
    if explicit:
        pos = (pos * 7 + 3).astype(np.int32)
    desc = B.make_desc(BF, hq, hkv, d)
    q = torch.full((rows, hq, d), float("nan"), dtype=BF, device=DEV)
    k = torch.full((rows, hkv, d), float("nan"), dtype=BF, device=DEV)
    v = torch.full((rows, hkv, d), float("nan"), dtype=BF, device=DEV)
    B.earn_qkv_rope_project(desc, x.to(DEV), wt(w), None if explicit else torch.from_numpy(cu).to(DEV),
                            torch.from_numpy(pos).to(DEV) if explicit else None, batch, q, k, v, workspace=ws)
    torch.cuda.synchronize()
    ref = O.qkv_project(W.to_f64(x), W.to_f64(w), hq, hkv, d, pos)
    check_attn(q, ref["q"], BF, "q")
    check_attn(k, ref["k"], BF, "k")
    check_attn(v, ref["v"], BF, "v")
    # rotation off: the plain product
    desc0 = B.make_desc(BF, hq, hkv, d, rope_base=0.0)
    B.earn_qkv_rope_project(desc0, x.to(DEV), wt(w), None, None, batch, q, k, v, workspace=ws)
    torch.cuda.synchronize()
    ref0 = O.qkv_project(W.to_f64(x), W.to_f64(w), hq, hkv, d, pos, rope_base=0.0)
    check_attn(q, ref0["q"], BF, "q without rotation")
    check_attn(k, ref0["k"], BF, "k without rotation")


@pytest.mark.parametrize("rows,k,n,act", [(300, 256, 512, 0), (1000, 4096, 136, 1), (7, 64, 8, 1), (513, 128, 1000, 0),
                                           (256, 1024, 128, 1), (40, 2048, 328, 1), (160, 4096, 256, 0)])
def test_linear_matches_oracle(rows, k, n, act, tile, ws):
    B = _B()
    g = torch.Generator().manual_seed(rows + k + n)
    x, w = rnd(g, rows, k), rnd(g, k, n, scale=k ** -0.5)
    out = torch.full((rows + 1, n), float("nan"), dtype=BF, device=DEV)
    B.earn_linear(x.to(DEV), wt(w), out[:rows], act, workspace=ws)
    torch.cuda.synchronize()
    ref = O.linear(W.to_f64(x), W.to_f64(w), act)
    got = out[:rows].cpu().double().numpy()
    assert np.isfinite(got).all() and torch.isnan(out[rows].float()).all()     # nothing written past the last row
    # row vectors against their norm, and element-wise against bf16 resolution at the scale of the row
    check_attn(got[:, None, :], ref[:, None, :], BF, "linear")
    assert (np.abs(got - ref) <= 2.0 ** -7 * np.maximum(np.abs(ref), np.abs(ref).max(axis=1, keepdims=True) * 0.05)).all()


def test_projection_argument_errors():
    B = _B()
    x = torch.zeros(8, 64, dtype=BF, device=DEV)
    w = torch.zeros(4 * 64, 64, dtype=BF, device=DEV)
    q, k = torch.zeros(8, 2, 64, dtype=BF, device=DEV), torch.zeros(8, 1, 64, dtype=BF, device=DEV)
    desc = B.make_desc(BF, 2, 1, 64)
    with pytest.raises(B.EarnError) as e:
        B.earn_qkv_rope_project(desc, x, w, None, None, 1, q, k, k.clone())     # rotation on, no positions at all
    assert e.value.code == B.EARN_ERR_INVALID_ARG
    with pytest.raises(B.EarnError) as e:
        B.earn_qkv_rope_project(B.make_desc(torch.float32, 2, 1, 64), x, w, None, torch.zeros(8, dtype=torch.int32, device=DEV), 1, q, k, k.clone())
    assert e.value.code == B.EARN_ERR_UNSUPPORTED
    with pytest.raises(B.EarnError) as e:
        B.earn_linear(torch.zeros(8, 96, dtype=BF, device=DEV), torch.zeros(64, 96, dtype=BF, device=DEV), torch.zeros(8, 64, dtype=BF, device=DEV))
    assert e.value.code == B.EARN_ERR_UNSUPPORTED and "multiple of 64" in str(e.value)
    with pytest.raises(B.EarnError) as e:
        B.earn_linear(x, w, torch.zeros(8, 256, dtype=BF, device=DEV), activation=5)
    assert e.value.code == B.EARN_ERR_INVALID_ARG


@pytest.mark.parametrize("hq,hkv,d,dm,lens", [(8, 2, 128, 256, [300, 64, 1000]), (14, 2, 64, 128, [17, 530, 3200])])
def test_projection_fed_path_matches_oracle(hq, hkv, d, dm, lens):
    """A full layer's attention fed by the projection (full length), the compaction of the HIDDEN rows, the
    register-focused layer projected from the gathered rows at their original positions, and a decode step whose q, k_new,
    v_new come from the projection of the new tokens' hidden rows: every attention call runs with rotation off."""
    B = _B()
    h, t = 4, 4
    r, rows, batch = h + t, sum(lens), len(lens)
    g = torch.Generator().manual_seed(rows + dm)
    ncol = (hq + 2 * hkv) * d
    x = rnd(g, rows, dm)
    w0, w1 = rnd(g, dm, ncol, scale=dm ** -0.5), rnd(g, dm, ncol, scale=dm ** -0.5)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    dcu = torch.from_numpy(cu).to(DEV)
    desc, desc0 = B.make_desc(BF, hq, hkv, d), B.make_desc(BF, hq, hkv, d, rope_base=0.0)
    dx = x.to(DEV)
    e = lambda n_, hh: torch.empty(n_, hh, d, dtype=BF, device=DEV)
    # layer 0: project, attend (no rotation pass, keys in place: no workspace)
    q0, k0, v0, o0 = e(rows, hq), e(rows, hkv), e(rows, hkv), e(rows, hq)
    B.earn_qkv_rope_project(desc, dx, wt(w0), dcu, None, batch, q0, k0, v0)
    assert B.earn_prefill_workspace_bytes(desc0, batch, rows, max(lens), False) == 0
    B.earn_prefill_attn(desc0, q0, k0, v0, dcu, None, batch, rows, max(lens), o0, None, None, None)
    # compaction of the hidden rows only; layer 1 projects from them at the original positions
    x_c = torch.empty(batch * r, dm, dtype=BF, device=DEV)
    idx, pos = (torch.empty(batch * r, dtype=torch.int32, device=DEV) for _ in range(2))
    cu_c = torch.empty(batch + 1, dtype=torch.int32, device=DEV)
    B.earn_compact_registers([dx], [x_c], dcu, batch, h, t, idx, pos, cu_c)
    q1, k1, v1, o1 = e(batch * r, hq), e(batch * r, hkv), e(batch * r, hkv), e(batch * r, hq)
    B.earn_qkv_rope_project(desc, x_c, wt(w1), None, pos, batch, q1, k1, v1)
    B.earn_prefill_attn(desc0, q1, k1, v1, cu_c, pos, batch, batch * r, r, o1, None, None, None)
    # decode step 0 of both layers: the new tokens' hidden rows, projected at position n_s
    S = batch
    xd = rnd(g, S, dm)
    q_pos, gen_len = (torch.empty(S, dtype=torch.int32, device=DEV) for _ in range(2))
    B.earn_decode_step_positions(dcu, None, S, batch, 0, q_pos, gen_len)
    outs = []
    for wl, kc, vc, scu, mlen in ((w0, k0, v0, dcu, max(lens)), (w1, k1, v1, cu_c, r)):
        dq, dk, dv = e(S, hq), e(S, hkv), e(S, hkv)
        B.earn_qkv_rope_project(desc, xd.to(DEV), wt(wl), None, q_pos, batch, dq, dk, dv)
        gk, gv = torch.zeros(S, 2, hkv, d, dtype=BF, device=DEV), torch.zeros(S, 2, hkv, d, dtype=BF, device=DEV)
        od = e(S, hq)
        ws = torch.empty(max(B.earn_decode_workspace_bytes(desc0, S, batch, mlen, 2), 256), dtype=torch.uint8, device=DEV)
        B.earn_decode_attn(desc0, dq, dk, dv, q_pos, kc, vc, scu, None, gk, gv, gen_len, 2, S, batch, mlen, od, ws)
        outs.append((od, gk))
    torch.cuda.synchronize()

    # oracle: the same steps in fp64 (projections rotated by the oracle, attention oracle with rotation off)
    f = W.to_f64
    pos_full = np.concatenate([np.arange(n) for n in lens]).astype(np.int32)
    p0 = O.qkv_project(f(x), f(w0), hq, hkv, d, pos_full)
    a0 = O.prefill_attn(p0["q"], p0["k"], p0["v"], cu, rope_base=0.0)
    check_attn(o0, a0["out"], BF, "layer 0 attention")
    check_attn(k0, p0["k"], BF, "layer 0 cache")
    comp = O.compact_registers(x.view(torch.int16).numpy(), cu, h, t)
    np.testing.assert_array_equal(idx.cpu().numpy(), comp["idx"])
    assert torch.equal(x_c.cpu().view(torch.int16), torch.from_numpy(comp["dst"]))
    xc64 = f(x)[comp["idx"]]
    p1 = O.qkv_project(xc64, f(w1), hq, hkv, d, comp["pos"])
    a1 = O.prefill_attn(p1["q"], p1["k"], p1["v"], comp["cu"], comp["pos"], rope_base=0.0)
    check_attn(o1, a1["out"], BF, "register layer attention")
    qp = np.asarray(lens, dtype=np.int32)
    for (od, gk), wl, pc, scu in ((outs[0], w0, p0, cu), (outs[1], w1, p1, comp["cu"])):
        pd = O.qkv_project(f(xd), f(wl), hq, hkv, d, qp)
        ogk, ogv = np.zeros((S, 2, hkv, d)), np.zeros((S, 2, hkv, d))
        rd = O.decode_attn(pd["q"], pd["k"], pd["v"], qp, pc["k"], pc["v"], scu, None, ogk, ogv, [0] * S, rope_base=0.0)
        check_attn(od, rd["out"], BF, "decode")
        check_attn(gk[:, 0], ogk[:, 0], BF, "appended key")


def test_full_size_projections_sampled_rows():
    """The headline workload's projection sizes (132096 rows, d_model 4096, d_ffn 11008, 32 + 2 x 8 heads of 128), in the
    256 x 256 tile form the library picks for them: sampled rows (tile corners, the last row, random rows) of the
    feed-forward product with SiLU and of the Q/K/V projection with rotation against the oracle."""
    B = _B()
    cfg = W.CONFIGS["long_beam"]
    w_ = W.Workload(cfg)
    rows, dm, df, hq, hkv, d = w_.total_tokens, 4096, 11008, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    g = torch.Generator(device=DEV).manual_seed(5)
    x = torch.randn(rows, dm, device=DEV, generator=g).to(BF)
    w_up = (torch.randn(df, dm, device=DEV, generator=g) * dm ** -0.5).to(BF)
    w_qkv = (torch.randn((hq + 2 * hkv) * d, dm, device=DEV, generator=g) * dm ** -0.5).to(BF)
    rng = np.random.default_rng(11)
    sample = sorted({0, 255, 256, 1023, 1024, rows - 257, rows - 1, *[int(r) for r in rng.integers(0, rows, size=24)]})
    xs = W.to_f64(x[sample].cpu())
    # feed-forward up-projection with SiLU
    hmid = torch.empty(rows, df, dtype=BF, device=DEV)
    B.earn_linear(x, w_up, hmid, 1, None)
    torch.cuda.synchronize()
    ref = O.linear(xs, W.to_f64(w_up.cpu()).T, 1)
    check_attn(hmid[sample].cpu()[:, None, :], ref[:, None, :], BF, "ffn up + SiLU, sampled rows")
    del hmid
    # Q/K/V projection with rotation at the tokens' positions
    pos = np.concatenate([np.arange(n) for n in w_.seq_lengths]).astype(np.int32)
    cu = torch.tensor(w_.cu_seqlens, dtype=torch.int32, device=DEV)
    q, k, v = (torch.empty(rows, h_, d, dtype=BF, device=DEV) for h_ in (hq, hkv, hkv))
    B.earn_qkv_rope_project(B.make_desc(BF, hq, hkv, d, 0.0, cfg.rope_base), x, w_qkv, cu, None, cfg.batch, q, k, v, None)
    torch.cuda.synchronize()
    ref = O.qkv_project(xs, W.to_f64(w_qkv.cpu()).T, hq, hkv, d, pos[sample], rope_base=cfg.rope_base)
    check_attn(q[sample], ref["q"], BF, "q, sampled rows")
    check_attn(k[sample], ref["k"], BF, "k, sampled rows")
    check_attn(v[sample], ref["v"], BF, "v, sampled rows")
