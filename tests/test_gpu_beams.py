"""Beam machinery against the oracle: top-k selection (bit-exact indices, one-chunk and two-phase forms), the ancestor
table, and whole beam-search decode loops in which the HIP path never copies a cache row (earn_decode_attn_beams reads
through the table) while the oracle follows the plain definition: every new beam takes a copy of its parent's cache."""
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


def gpu_topk(B, bs, lp, batch, beams, vocab):
    parent = torch.full((batch * beams,), -7, dtype=torch.int32, device=DEV)
    token = torch.full_like(parent, -7)
    score = torch.full((batch * beams,), float("nan"), dtype=torch.float32, device=DEV)
    B.earn_beam_topk(None if bs is None else torch.from_numpy(bs).to(DEV), torch.from_numpy(lp).to(DEV), batch, beams,
                     vocab, parent, token, score)
    torch.cuda.synchronize()
    return parent.cpu().numpy(), token.cpu().numpy(), score.cpu().numpy()


@pytest.mark.parametrize("batch,beams,vocab", [(16, 20, 256), (3, 20, 409), (2, 20, 32000), (5, 1, 1000), (1, 64, 128),
                                               (4, 7, 1), (2, 3, 8192)])
def test_beam_topk_is_bit_exact(batch, beams, vocab):
    B = _B()
    rng = np.random.default_rng(batch * 1000 + vocab)
    lp = rng.standard_normal((batch * beams, vocab)).astype(np.float32)
    lp = np.round(lp * 8) / 8                       # many exact ties: the order among equals is part of the result
    lp[rng.random(lp.shape) < 0.01] = -np.inf
    if vocab > 4:
        lp[0, 1] = np.nan
        lp[-1, -3:] = 50.0                          # ties at the very top, at the end of the last chunk
    bs = (np.round(rng.standard_normal(batch * beams) * 4) / 4).astype(np.float32)
    ref = O.beam_topk(bs, lp, batch, beams, vocab)
    parent, token, score = gpu_topk(B, bs, lp, batch, beams, vocab)
    np.testing.assert_array_equal(parent, ref["parent"])
    np.testing.assert_array_equal(token, ref["token"])
    np.testing.assert_array_equal(score, ref["score"])
    if vocab == 256:
        p2, t2, s2 = gpu_topk(B, None, lp, batch, beams, vocab)
        r2 = O.beam_topk(None, lp, batch, beams, vocab)
        np.testing.assert_array_equal(p2, r2["parent"])
        np.testing.assert_array_equal(t2, r2["token"])


def test_beam_argument_errors_and_limits():
    B = _B()
    z = torch.zeros(4, 8, device=DEV)
    o = torch.zeros(4, dtype=torch.int32, device=DEV)
    s = torch.zeros(4, device=DEV)
    with pytest.raises(B.EarnError) as e:
        B.earn_beam_topk(None, z, 0, 4, 8, o, o, s)
    assert e.value.code == B.EARN_ERR_INVALID_ARG
    with pytest.raises(B.EarnError) as e:
        B.earn_beam_topk(None, z, 1, 65, 8, o, o, s)
    assert e.value.code == B.EARN_ERR_UNSUPPORTED
    assert B.earn_beam_topk_workspace_bytes(16, 20, 256) == 0
    assert B.earn_beam_topk_workspace_bytes(2, 20, 32000) == 2 * 79 * 20 * 8
    with pytest.raises(B.EarnError) as e:
        B.lib()  # a two-phase problem without workspace
        B._check(B.lib().earn_beam_topk(None, B._ptr(z), 2, 20, 32000, B._ptr(o), B._ptr(o), B._ptr(s), None, 0, None))
    assert e.value.code == B.EARN_ERR_WORKSPACE_TOO_SMALL
    with pytest.raises(B.EarnError):
        B.earn_beam_reorder(o, o, o, 4, 1, 0)       # aliased tables
    with pytest.raises(B.EarnError):
        B.earn_beam_reorder(o, None, torch.zeros(4, 2, dtype=torch.int32, device=DEV), 4, 2, 2)   # step outside the cache


def test_beam_reorder_table():
    B = _B()
    S, cap = 6, 4
    src0 = torch.empty(S, cap, dtype=torch.int32, device=DEV)
    parent0 = torch.tensor([0, 0, 1, 3, 5, 5], dtype=torch.int32, device=DEV)
    B.earn_beam_reorder(parent0, None, src0, S, cap, 0)
    torch.cuda.synchronize()
    assert src0.tolist() == [[0, 0, 0, 0], [0, 1, 1, 1], [1, 2, 2, 2], [3, 3, 3, 3], [5, 4, 4, 4], [5, 5, 5, 5]]
    src1 = torch.empty_like(src0)
    parent1 = torch.tensor([2, 1, 1, 4, 4, 3], dtype=torch.int32, device=DEV)
    B.earn_beam_reorder(parent1, src0, src1, S, cap, 1)
    torch.cuda.synchronize()
    # stream 0 now descends from old stream 2, whose step-0 row sits in stream 1's slot
    assert src1.tolist() == [[1, 2, 0, 0], [0, 1, 1, 1], [0, 1, 2, 2], [5, 4, 3, 3], [5, 4, 4, 4], [3, 3, 5, 5]]


BEAM_CASES = [
    # dtype, hq, hkv, d, shared lengths, beams, steps, vocab
    (BF, 32, 8, 128, [64, 300], 20, 4, 256),        # the paper's beam width: 80 query rows per cache, matrix-core kernel
    (BF, 8, 8, 64, [33, 16, 700], 4, 5, 50),        # vector kernel (one query head per kv head, short caches)
    (BF, 14, 2, 64, [1000, 130], 3, 3, 1000),       # key splits + combine
    (F32, 4, 2, 64, [40, 9], 5, 4, 16),
]


@pytest.mark.parametrize("dtype,hq,hkv,d,slens,beams,steps,vocab", BEAM_CASES)
def test_beam_search_decode_loop_matches_oracle(dtype, hq, hkv, d, slens, beams, steps, vocab):
    B = _B()
    batch, S = len(slens), len(slens) * beams
    g = torch.Generator().manual_seed(sum(slens) + beams)
    rnd = lambda *s: torch.randn(*s, generator=g).to(dtype)
    cu = np.concatenate([[0], np.cumsum(slens)]).astype(np.int32)
    s2s = [u // beams for u in range(S)]
    sk, sv = rnd(int(cu[-1]), hkv, d), rnd(int(cu[-1]), hkv, d)
    desc = B.make_desc(dtype, hq, hkv, d)
    dev = lambda x: x.to(DEV)
    i32 = lambda x: torch.tensor(list(x), dtype=torch.int32, device=DEV)
    d_sk, d_sv, d_cu, d_s2s = dev(sk), dev(sv), i32(cu), i32(s2s)
    gk = torch.zeros(S, steps, hkv, d, dtype=dtype, device=DEV)
    gv = torch.zeros_like(gk)
    src = [torch.zeros(S, steps, dtype=torch.int32, device=DEV) for _ in range(2)]
    have_src = False
    ws = torch.empty(max(B.earn_decode_workspace_bytes(desc, S, batch, max(slens), steps), 256), dtype=torch.uint8, device=DEV)
    q_pos, gen_len = (torch.zeros(S, dtype=torch.int32, device=DEV) for _ in range(2))
    parent, token = (torch.zeros(S, dtype=torch.int32, device=DEV) for _ in range(2))
    scores = torch.zeros(S, dtype=torch.float32, device=DEV)
    # the oracle's state: every stream owns a full copy of its history
    o_gk, o_gv = np.zeros((S, steps, hkv, d)), np.zeros((S, steps, hkv, d))
    o_scores = np.zeros(S, dtype=np.float32)
    rng = np.random.default_rng(beams)
    for step in range(steps):
        q, kn, vn = rnd(S, hq, d), rnd(S, hkv, d), rnd(S, hkv, d)
        B.earn_decode_step_positions(d_cu, d_s2s, S, batch, step, q_pos, gen_len)
        out = torch.full((S, hq, d), float("nan"), dtype=dtype, device=DEV)
        B.earn_decode_attn_beams(desc, dev(q), dev(kn), dev(vn), q_pos, d_sk, d_sv, d_cu, d_s2s, gk, gv, gen_len,
                                 src[step % 2] if have_src else None, steps, S, batch, max(slens), out, ws)
        torch.cuda.synchronize()
        ref = O.decode_attn(W.to_f64(q), W.to_f64(kn), W.to_f64(vn), [slens[s2s[u]] + step for u in range(S)],
                            W.to_f64(sk), W.to_f64(sv), cu, s2s, o_gk, o_gv, [step] * S)
        check_attn(out, ref["out"], dtype, f"step {step}")
        # selection: random log-probabilities with ties; beams are shuffled, some die, some fork
        lp = (np.round(rng.standard_normal((S, vocab)) * 4) / 4).astype(np.float32)
        sel = O.beam_topk(o_scores, lp, batch, beams, vocab)
        B.earn_beam_topk(scores, torch.from_numpy(lp).to(DEV), batch, beams, vocab, parent, token, scores_new := torch.empty_like(scores))
        torch.cuda.synchronize()
        np.testing.assert_array_equal(parent.cpu().numpy(), sel["parent"])
        np.testing.assert_array_equal(token.cpu().numpy(), sel["token"])
        np.testing.assert_array_equal(scores_new.cpu().numpy(), sel["score"])
        scores, o_scores = scores_new, sel["score"]
        B.earn_beam_reorder(parent, src[step % 2] if have_src else None, src[(step + 1) % 2], S, steps, step)
        have_src = True
        O.beam_reorder_caches(sel["parent"], o_gk, o_gv)
    assert len(set(sel["parent"].tolist())) < S       # the loop did fork and drop beams
