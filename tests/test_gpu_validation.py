"""Debug validation of the preconditions that live in device memory (earn_set_validation), and what the kernels guard
without it.

With validation on, a call whose device arrays break a precondition returns EARN_ERR_INVALID_ARG BEFORE any kernel is
launched: the tests assert the code and that the outputs still hold their sentinel.  No kernel ever runs on bad input
here.  The last test runs the matrix-core kernels on VALID inputs whose neighbouring rows in memory hold NaN: rows past
the end of a sequence must reach the kernels as zeros, whatever lies behind them.
"""
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


@pytest.fixture
def validating():
    B = _B()
    old = B.earn_set_validation(True)
    yield B
    B.earn_set_validation(old)


def i32(x):
    return torch.tensor(list(x), dtype=torch.int32, device=DEV)


def expect_invalid(B, fn, needle):
    with pytest.raises(B.EarnError) as e:
        fn()
    assert e.value.code == B.EARN_ERR_INVALID_ARG, str(e.value)
    assert needle in str(e.value), str(e.value)


def test_prefill_validation(validating):
    B = validating
    hq, hkv, d, T = 4, 2, 64, 96
    q = torch.zeros(T, hq, d, dtype=BF, device=DEV)
    k = torch.zeros(T, hkv, d, dtype=BF, device=DEV)
    out = torch.full_like(q, 7.0)
    krot = torch.full_like(k, 7.0)
    desc = B.make_desc(BF, hq, hkv, d)
    call = lambda cu, pos=None, maxlen=64: B.earn_prefill_attn(desc, q, k, k, i32(cu), pos, len(cu) - 1, T, maxlen, out,
                                                                krot, None, None)
    expect_invalid(B, lambda: call([0, 64, 32, 96]), "decreases")
    expect_invalid(B, lambda: call([1, 64, 96]), "must be 0")
    expect_invalid(B, lambda: call([0, 64, 95]), "expected 96")
    expect_invalid(B, lambda: call([0, 90, 96]), "more than the bound")
    expect_invalid(B, lambda: call([0, 64, 96], pos=i32([0] * 95 + [-3])), "positions[95]")
    torch.cuda.synchronize()
    assert (out == 7.0).all() and (krot == 7.0).all()      # nothing was launched
    call([0, 64, 96])                                       # a valid call goes through
    torch.cuda.synchronize()
    assert not (out == 7.0).any()


def test_compaction_validation(validating):
    B = validating
    src = torch.zeros(40, 32, dtype=torch.uint8, device=DEV)
    dst = torch.full((8, 32), 9, dtype=torch.uint8, device=DEV)
    idx = torch.full((8,), -5, dtype=torch.int32, device=DEV)
    call = lambda cu, h=2, t=2: B.earn_compact_registers([src], [dst], i32(cu), 2, h, t, idx, None, None)
    expect_invalid(B, lambda: call([0, 3, 40]), "fewer than h + t")
    expect_invalid(B, lambda: call([0, 30, 20]), "decreases")
    torch.cuda.synchronize()
    assert (dst == 9).all() and (idx == -5).all()
    call([0, 4, 40])
    torch.cuda.synchronize()
    assert idx.tolist() == [0, 1, 2, 3, 4, 5, 38, 39]


def test_decode_validation(validating):
    B = validating
    hq, hkv, d, S, batch, gen_cap = 4, 2, 64, 4, 2, 3
    z = lambda *s: torch.zeros(*s, dtype=BF, device=DEV)
    q, kn, sk = z(S, hq, d), z(S, hkv, d), z(50, hkv, d)
    gk, gv = torch.full((S, gen_cap, hkv, d), 3.0, dtype=BF, device=DEV), torch.full((S, gen_cap, hkv, d), 3.0, dtype=BF, device=DEV)
    out = torch.full_like(q, 7.0)
    desc = B.make_desc(BF, hq, hkv, d)
    ws = torch.empty(max(B.earn_decode_workspace_bytes(desc, S, batch, 40, gen_cap), 256), dtype=torch.uint8, device=DEV)

    def call(cu=(0, 40, 50), s2s=(0, 0, 1, 1), glen=(0, 1, 2, 0), qpos=(40, 41, 12, 10), maxlen=40):
        B.earn_decode_attn(desc, q, kn, kn, i32(qpos), sk, sk, i32(cu), i32(s2s), gk, gv, i32(glen), gen_cap, S, batch,
                           maxlen, out, ws)

    expect_invalid(B, lambda: call(glen=(0, 1, 3, 0)), "gen_len[2]")
    expect_invalid(B, lambda: call(glen=(-1, 1, 2, 0)), "gen_len[0]")
    expect_invalid(B, lambda: call(s2s=(0, 0, 2, 1)), "stream_to_seq[2]")
    expect_invalid(B, lambda: call(s2s=(0, -1, 1, 1)), "stream_to_seq[1]")
    expect_invalid(B, lambda: call(cu=(0, 45, 50)), "more than the bound")
    expect_invalid(B, lambda: call(cu=(0, 40, 30)), "decreases")
    expect_invalid(B, lambda: call(qpos=(40, 41, -1, 10)), "q_pos[2]")
    torch.cuda.synchronize()
    assert (out == 7.0).all() and (gk == 3.0).all() and (gv == 3.0).all()
    call()
    torch.cuda.synchronize()
    assert not (out == 7.0).any()


def test_decode_validation_counts_streams_per_sequence(validating):
    B = validating
    hq, hkv, d, batch, gen_cap = 2, 2, 64, 30, 1
    S = 1025 + 28                      # the host cannot tell from n_streams and batch alone (S <= 1024 * batch)
    z = lambda *s: torch.zeros(*s, dtype=BF, device=DEV)
    q, kn, sk = z(S, hq, d), z(S, hkv, d), z(batch * 200, hkv, d)
    gk = z(S, gen_cap, hkv, d)
    out = torch.full_like(q, 7.0)
    desc = B.make_desc(BF, hq, hkv, d)
    ws = torch.empty(max(B.earn_decode_workspace_bytes(desc, S, batch, 200, gen_cap), 256), dtype=torch.uint8, device=DEV)
    s2s = [0] * 1025 + list(range(1, 29))
    expect_invalid(B, lambda: B.earn_decode_attn(desc, q, kn, kn, i32([200] * S), sk, sk, i32(range(0, 200 * batch + 1, 200)),
                                                 i32(s2s), gk, gk.clone(), i32([0] * S), gen_cap, S, batch, 200, out, ws),
                   "more than 1024 streams")
    torch.cuda.synchronize()
    assert (out == 7.0).all()


def test_register_rows_validation(validating):
    B = validating
    hq, hkv, d, T, r = 4, 2, 64, 100, 4
    z = lambda *s: torch.zeros(*s, dtype=BF, device=DEV)
    k = z(T, hkv, d)
    q_rows = z(2 * r, hq, d)
    out = torch.full_like(q_rows, 7.0)
    krot = torch.full_like(k, 7.0)
    desc = B.make_desc(BF, hq, hkv, d)
    ws = torch.empty(max(B.earn_prefill_register_rows_workspace_bytes(desc, 2, 60, r), 256), dtype=torch.uint8, device=DEV)
    call = lambda pos, cu=(0, 60, 100): B.earn_prefill_register_rows(desc, q_rows, k, k, i32(cu), i32(pos), 2, T, 60, r,
                                                                       out, krot, ws)
    expect_invalid(B, lambda: call([0, 1, 58, 60, 0, 1, 38, 39]), "row_pos[3]")     # past the sequence
    expect_invalid(B, lambda: call([0, 1, 58, 59, 0, 5, 5, 39]), "row_pos[6]")      # not ascending
    expect_invalid(B, lambda: call([0, 1, 58, 59, 0, 1, 38, 39], cu=(0, 60, 99)), "expected 100")
    torch.cuda.synchronize()
    assert (out == 7.0).all() and (krot == 7.0).all()
    call([0, 1, 58, 59, 0, 1, 38, 39])
    torch.cuda.synchronize()
    assert not (out == 7.0).any()


def test_validation_is_off_by_default_and_switches_back():
    B = _B()
    assert B.earn_set_validation(True) is False
    assert B.earn_set_validation(False) is True
    assert B.earn_set_validation(False) is False


def test_tuning_keys():
    B = _B()
    B.earn_set_tuning("decode_vec_waves", 2)
    B.earn_set_tuning("decode_vec_waves", 0)
    with pytest.raises(B.EarnError) as e:
        B.earn_set_tuning("no_such_key", 1)
    assert e.value.code == B.EARN_ERR_INVALID_ARG


# --------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("d", [64, 128])
def test_rows_behind_a_sequence_reach_the_kernels_as_zeros(d):
    """Sequences A and B, each followed in memory by 64 guard rows of NaN (packed as sequences of their own, whose
    outputs nobody reads).  A K/V tile that reaches past the end of A or B must see zeros there: 0 x NaN in the second
    product would poison the output otherwise.  The last guard also keeps the tail tile of the last real sequence
    inside the allocation.  Outputs must be finite, match the oracle, and equal bit for bit what the same sequences
    give without guards."""
    B = _B()
    hq, hkv, h, t = 8, 2, 4, 4
    lens = [300, 64, 1111, 64]                 # A, guard, B, guard
    real = [0, 2]
    T, batch, r = sum(lens), len(lens), h + t
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    g = torch.Generator().manual_seed(5 + d)
    rnd = lambda *s: torch.randn(*s, generator=g).to(BF)
    q, k, v = rnd(T, hq, d), rnd(T, hkv, d), rnd(T, hkv, d)
    for s in (1, 3):
        k[cu[s]:cu[s + 1]] = float("nan")
        v[cu[s]:cu[s + 1]] = float("nan")
    rows_real = np.concatenate([np.arange(cu[s], cu[s + 1]) for s in real])
    cu2 = np.concatenate([[0], np.cumsum([lens[s] for s in real])]).astype(np.int32)
    q2, k2, v2 = (x[torch.from_numpy(rows_real)].contiguous() for x in (q, k, v))
    ref = O.prefill_attn(W.to_f64(q2), W.to_f64(k2), W.to_f64(v2), cu2)
    desc = B.make_desc(BF, hq, hkv, d)
    dev = lambda x: x.to(DEV)

    # prefill (128-row workgroups here; the tile staging is shared by all matrix-core kernels)
    def prefill(qq, kk, vv, cc):
        out = torch.empty(qq.shape, dtype=BF, device=DEV)
        kr = torch.empty(kk.shape, dtype=BF, device=DEV)
        ln = np.diff(cc)
        B.earn_prefill_attn(desc, dev(qq), dev(kk), dev(vv), torch.from_numpy(cc).to(DEV), None, len(ln), int(cc[-1]),
                            int(ln.max()), out, kr, None, None)
        torch.cuda.synchronize()
        return out.cpu(), kr.cpu()

    out_g, kr_g = prefill(q, k, v, cu)
    out_p, kr_p = prefill(q2, k2, v2, cu2)
    got = out_g[torch.from_numpy(rows_real)]
    assert torch.isfinite(got.float()).all()
    check_attn(got, ref["out"], BF, "prefill next to NaN rows")
    assert torch.equal(got, out_p)

    # the register rows of the same layer
    comp = O.compact_registers(None, cu, h, t)
    comp2 = O.compact_registers(None, cu2, h, t)

    def rows(qq, kk, vv, cc, cmp_):
        ln = np.diff(cc)
        q_rows = qq[torch.from_numpy(cmp_["idx"]).long()].contiguous()
        out = torch.empty(q_rows.shape, dtype=BF, device=DEV)
        kr = torch.empty(kk.shape, dtype=BF, device=DEV)
        ws = torch.empty(max(B.earn_prefill_register_rows_workspace_bytes(desc, len(ln), int(ln.max()), r), 256),
                         dtype=torch.uint8, device=DEV)
        B.earn_prefill_register_rows(desc, dev(q_rows), dev(kk), dev(vv), torch.from_numpy(cc).to(DEV),
                                     torch.from_numpy(cmp_["pos"]).to(DEV), len(ln), int(cc[-1]), int(ln.max()), r, out,
                                     kr, ws)
        torch.cuda.synchronize()
        return out.cpu()

    rr_g = rows(q, k, v, cu, comp).reshape(batch, r, hq, d)[real].reshape(-1, hq, d)
    rr_p = rows(q2, k2, v2, cu2, comp2)
    assert torch.isfinite(rr_g.float()).all()
    check_attn(rr_g, ref["out"][comp2["idx"]], BF, "register rows next to NaN rows")
    assert torch.equal(rr_g, rr_p)

    # a decode step over the same caches (rotated keys from the prefill), beams on the real sequences only
    beams, gen_cap = 3, 2
    s2s_g = [s for s in real for _ in range(beams)]
    s2s_p = [i for i in range(len(real)) for _ in range(beams)]
    S = len(s2s_g)
    dq, dk, dv = rnd(S, hq, d), rnd(S, hkv, d), rnd(S, hkv, d)
    gk0, gv0 = rnd(S, gen_cap, hkv, d), rnd(S, gen_cap, hkv, d)
    glen = [u % gen_cap for u in range(S)]

    def decode(kr, vv, cc, s2s, lens_):
        qpos = [lens_[s2s[u]] + glen[u] for u in range(S)]
        out = torch.empty(S, hq, d, dtype=BF, device=DEV)
        ws = torch.empty(max(B.earn_decode_workspace_bytes(desc, S, len(lens_), max(lens_), gen_cap), 256),
                         dtype=torch.uint8, device=DEV)
        B.earn_decode_attn(desc, dev(dq), dev(dk), dev(dv), i32(qpos), dev(kr), dev(vv), torch.from_numpy(cc).to(DEV),
                           i32(s2s), dev(gk0), dev(gv0), i32(glen), gen_cap, S, len(lens_), max(lens_), out, ws)
        torch.cuda.synchronize()
        return out.cpu(), qpos

    kr_g_nan = kr_g.clone()
    for s in (1, 3):
        kr_g_nan[cu[s]:cu[s + 1]] = float("nan")
    dec_g, qpos = decode(kr_g_nan, v, cu, s2s_g, lens)
    dec_p, _ = decode(kr_p, v2, cu2, s2s_p, [lens[s] for s in real])
    assert torch.isfinite(dec_g.float()).all()
    assert torch.equal(dec_g, dec_p)
    ogk, ogv = W.to_f64(gk0), W.to_f64(gv0)
    dref = O.decode_attn(W.to_f64(dq), W.to_f64(dk), W.to_f64(dv), qpos, W.to_f64(kr_p), W.to_f64(v2), cu2, s2s_p, ogk,
                         ogv, glen)
    check_attn(dec_g, dref["out"], BF, "decode next to NaN rows")
