"""Pins for the CPU oracle: everything here checks oracle/ against something other than itself.

Each pin is chosen so that a plausible mistake (dropped term, wrong sign or index, transposed operand,
renumbered positions) fails at least one test.  The references used are: a library routine (torch SDPA in fp64),
a dense-mask NumPy formulation with rotary embedding done as a complex multiplication, closed forms, brute
force on tiny inputs, and the worked example of the paper's efficiency analysis (tests/golden/).
"""
import os

import numpy as np
import pytest
import torch

from oracle import earn_oracle as O
from oracle import pipeline as OP

RNG = np.random.default_rng(20250700715)
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------------------------
# independent references (NumPy, dense masks)
# ----------------------------------------------------------------------------------------------
def rope_complex(x, pos, base):
    """Rotary embedding as multiplication by e^{i p theta} on the pairs (x_i, x_{i+d/2})."""
    d = x.shape[-1]
    z = x[..., : d // 2] + 1j * x[..., d // 2:]
    theta = base ** (-np.arange(d // 2) * 2.0 / d)
    rot = np.exp(1j * np.asarray(pos, dtype=np.float64)[:, None, None] * theta[None, None, :])
    z = z * rot
    return np.concatenate([z.real, z.imag], axis=-1)


def dense_masked_attention(q, k, v, mask, group):
    """softmax(q k^T / sqrt(d) + mask) v for one sequence; q [n,Hq,d], k/v [n,Hkv,d], mask [n,n] bool."""
    n, hq, d = q.shape
    out = np.zeros_like(q)
    for a in range(hq):
        c = a // group
        s = q[:, a, :] @ k[:, c, :].T / np.sqrt(d)
        s = np.where(mask, s, -np.inf)
        s = s - s.max(axis=1, keepdims=True)
        p = np.exp(s)
        p = p / p.sum(axis=1, keepdims=True)
        out[:, a, :] = p @ v[:, c, :]
    return out


def rand_batch(lens, hq, hkv, d):
    T = int(sum(lens))
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    return (RNG.standard_normal((T, hq, d)), RNG.standard_normal((T, hkv, d)), RNG.standard_normal((T, hkv, d)), cu)


# ----------------------------------------------------------------------------------------------
# rotary embedding
# ----------------------------------------------------------------------------------------------
def test_rope_matches_complex_rotation():
    x = RNG.standard_normal((37, 3, 64))
    pos = RNG.integers(0, 9000, size=37)
    np.testing.assert_allclose(O.rope(x, pos, 10000.0), rope_complex(x, pos, 10000.0), rtol=0, atol=1e-10)  # angle ~ 9e3 rad x 1 ulp of theta


def test_rope_identity_at_zero_and_norm_preserving():
    x = RNG.standard_normal((5, 2, 128))
    np.testing.assert_array_equal(O.rope(x, np.zeros(5, dtype=np.int32)), x)
    y = O.rope(x, np.array([1, 77, 500, 8255, 8263]))
    np.testing.assert_allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-13)
    assert np.abs(y - x).max() > 0.1


def test_rope_known_quarter_turn():
    # d = 2: theta_0 = 1, so position p rotates the pair by p radians.
    x = np.array([[[1.0, 0.0]]])
    y = O.rope(x, np.array([1]), 10000.0)
    np.testing.assert_allclose(y[0, 0], [np.cos(1.0), np.sin(1.0)], atol=1e-15)
    # d = 4: second pair turns by base^(-1/2) per position.
    x = np.array([[[0.0, 1.0, 0.0, 0.0]]])
    y = O.rope(x, np.array([3]), 100.0)
    np.testing.assert_allclose(y[0, 0], [0.0, np.cos(0.3), 0.0, np.sin(0.3)], atol=1e-15)


def test_rope_disabled():
    x = RNG.standard_normal((4, 2, 8))
    np.testing.assert_array_equal(O.rope(x, np.arange(4), 0.0), x)


# ----------------------------------------------------------------------------------------------
# prefill attention (Eq. 3)
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("hq,hkv,d", [(4, 4, 64), (6, 2, 32), (14, 2, 64)])
def test_prefill_equals_library_sdpa_without_rope(hq, hkv, d):
    lens = [1, 17, 40]
    q, k, v, cu = rand_batch(lens, hq, hkv, d)
    res = O.prefill_attn(q, k, v, cu, rope_base=0.0)
    for s in range(len(lens)):
        sl = slice(cu[s], cu[s + 1])
        tq = torch.from_numpy(q[sl]).permute(1, 0, 2)[None]
        tk = torch.from_numpy(np.repeat(k[sl], hq // hkv, axis=1)).permute(1, 0, 2)[None]
        tv = torch.from_numpy(np.repeat(v[sl], hq // hkv, axis=1)).permute(1, 0, 2)[None]
        ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).numpy()
        np.testing.assert_allclose(res["out"][sl], ref, rtol=0, atol=1e-12)


def test_explicit_softmax_scale_equals_rescaled_queries_and_library_sdpa():
    """Eq. 3 with the factor 1/sqrt(d) replaced by an explicit scale s.  Scores are linear in q (the rotation is
    linear too), so scale s on q equals the default scale on q * s * sqrt(d); and without rotation the library
    routine takes the same scale directly.  Prefill and decode take the explicit branch alike."""
    lens, hq, hkv, d, s_ = [1, 17, 40], 6, 2, 16, 0.37
    q, k, v, cu = rand_batch(lens, hq, hkv, d)
    res = O.prefill_attn(q, k, v, cu, scale=s_, rope_base=10000.0)
    same = O.prefill_attn(q * (s_ * np.sqrt(d)), k, v, cu, rope_base=10000.0)
    np.testing.assert_allclose(res["out"], same["out"], rtol=0, atol=1e-12)
    np.testing.assert_allclose(res["lse"], same["lse"], rtol=0, atol=1e-12)
    assert np.abs(res["out"] - O.prefill_attn(q, k, v, cu, rope_base=10000.0)["out"]).max() > 1e-3  # it is not ignored
    plain = O.prefill_attn(q, k, v, cu, scale=s_, rope_base=0.0)
    for s in range(len(lens)):
        sl = slice(cu[s], cu[s + 1])
        tq = torch.from_numpy(q[sl]).permute(1, 0, 2)[None]
        tk = torch.from_numpy(np.repeat(k[sl], hq // hkv, axis=1)).permute(1, 0, 2)[None]
        tv = torch.from_numpy(np.repeat(v[sl], hq // hkv, axis=1)).permute(1, 0, 2)[None]
        ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=s_)[0]
        np.testing.assert_allclose(plain["out"][sl], ref.permute(1, 0, 2).numpy(), rtol=0, atol=1e-12)
    # decode step
    S, gen_cap = 3, 2
    dq, dk, dv = RNG.standard_normal((S, hq, d)), RNG.standard_normal((S, hkv, d)), RNG.standard_normal((S, hkv, d))
    args = lambda qq: (qq, dk, dv, [l + 1 for l in lens], res["k_rot"], v, cu, None)
    gk1, gv1 = np.zeros((S, gen_cap, hkv, d)), np.zeros((S, gen_cap, hkv, d))
    gk2, gv2 = gk1.copy(), gv1.copy()
    a = O.decode_attn(*args(dq), gk1, gv1, [0, 1, 0], scale=s_)
    b = O.decode_attn(*args(dq * (s_ * np.sqrt(d))), gk2, gv2, [0, 1, 0])
    np.testing.assert_allclose(a["out"], b["out"], rtol=0, atol=1e-12)


def test_prefill_with_rope_equals_dense_mask_reference():
    lens = [23, 9]
    q, k, v, cu = rand_batch(lens, 4, 2, 16)
    res = O.prefill_attn(q, k, v, cu, rope_base=10000.0)
    for s in range(2):
        sl = slice(cu[s], cu[s + 1])
        n = lens[s]
        pos = np.arange(n)
        qr, kr = rope_complex(q[sl], pos, 10000.0), rope_complex(k[sl], pos, 10000.0)
        ref = dense_masked_attention(qr, kr, v[sl], np.tril(np.ones((n, n), dtype=bool)), 2)
        np.testing.assert_allclose(res["out"][sl], ref, rtol=0, atol=1e-12)
        np.testing.assert_allclose(res["k_rot"][sl], kr, rtol=0, atol=1e-12)


def test_softmax_rows_sum_to_one_and_probs_are_causal():
    lens = [31, 50]
    q, k, v, cu = rand_batch(lens, 3, 3, 32)
    res = O.prefill_attn(q * 3.0, k * 3.0, v, cu, want_probs=(1, 2))
    assert np.abs(res["rowsum"] - 1.0).max() < 1e-12
    p = res["probs"]
    assert p.shape == (50, 50)
    assert np.abs(p.sum(axis=1) - 1.0).max() < 1e-12
    assert np.all(np.triu(p, 1) == 0.0) and np.all(p >= 0.0)
    # the probabilities reproduce the output and the log-sum-exp
    sl = slice(cu[1], cu[2])
    np.testing.assert_allclose(p @ v[sl, 2, :], res["out"][sl, 2, :], atol=1e-12)
    kr = res["k_rot"][sl, 2, :]
    qr = O.rope(q[sl] * 3.0, np.arange(50))[:, 2, :]
    s = np.where(np.tril(np.ones((50, 50), dtype=bool)), qr @ kr.T / np.sqrt(32), -np.inf)
    lse = np.log(np.exp(s - s.max(1, keepdims=True)).sum(1)) + s.max(1)
    np.testing.assert_allclose(res["lse"][sl, 2], lse, atol=1e-12)


def test_closed_forms():
    lens = [12, 20]
    q, k, v, cu = rand_batch(lens, 4, 2, 16)
    # first token attends to itself only
    res = O.prefill_attn(q, k, v, cu)
    for s in range(2):
        for a in range(4):
            np.testing.assert_allclose(res["out"][cu[s], a], v[cu[s], a // 2], atol=1e-14)
    # K == 0: uniform probabilities -> running mean of V
    res0 = O.prefill_attn(q, np.zeros_like(k), v, cu)
    for s in range(2):
        run = np.cumsum(v[cu[s]:cu[s + 1]], axis=0) / np.arange(1, lens[s] + 1)[:, None, None]
        np.testing.assert_allclose(res0["out"][cu[s]:cu[s + 1]], np.repeat(run, 2, axis=1), atol=1e-13)
    # V rows all equal to c: output is c
    c = RNG.standard_normal((1, 2, 16))
    resc = O.prefill_attn(q, k, np.broadcast_to(c, v.shape).copy(), cu)
    np.testing.assert_allclose(resc["out"], np.broadcast_to(np.repeat(c, 2, axis=1), q.shape), atol=1e-13)


def test_gqa_equals_mha_on_repeated_kv_and_explicit_map():
    lens = [15, 7]
    q, k, v, cu = rand_batch(lens, 6, 2, 16)
    g = O.prefill_attn(q, k, v, cu)["out"]
    m = O.prefill_attn(q, np.repeat(k, 3, axis=1), np.repeat(v, 3, axis=1), cu)["out"]
    np.testing.assert_allclose(g, m, atol=1e-13)
    perm = [1, 0, 1, 0, 0, 1]
    e = O.prefill_attn(q, k, v, cu, q_to_kv=perm)["out"]
    m2 = O.prefill_attn(q, k[:, perm], v[:, perm], cu)["out"]
    np.testing.assert_allclose(e, m2, atol=1e-13)


def test_relative_position_property_and_negative_pin():
    n, h, t = 40, 3, 2
    q, k, v, cu = rand_batch([n], 2, 2, 32)
    base = O.prefill_attn(q, k, v, cu, positions=np.arange(n))["out"]
    shifted = O.prefill_attn(q, k, v, cu, positions=np.arange(n) + 1234)["out"]
    np.testing.assert_allclose(base, shifted, atol=1e-9)
    # renumbering the kept suffix registers to h..r-1 instead of their original positions must change the result
    keep = list(range(h)) + list(range(n - t, n))
    cu_c = np.array([0, h + t], dtype=np.int32)
    orig = O.prefill_attn(q[keep], k[keep], v[keep], cu_c, positions=np.array(keep))["out"]
    renum = O.prefill_attn(q[keep], k[keep], v[keep], cu_c, positions=np.arange(h + t))["out"]
    assert np.abs(orig - renum).max() > 1e-3


def test_row_selection_computes_the_same_rows():
    lens = [30, 11]
    q, k, v, cu = rand_batch(lens, 2, 1, 16)
    full = O.prefill_attn(q, k, v, cu)
    sel = np.zeros(41, dtype=np.uint8)
    sel[[0, 7, 29, 30, 40]] = 1
    part = O.prefill_attn(q, k, v, cu, row_sel=sel)
    np.testing.assert_array_equal(part["out"][sel == 1], full["out"][sel == 1])
    assert np.isnan(part["out"][sel == 0]).all()


# ----------------------------------------------------------------------------------------------
# register compaction
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("h,t", [(2, 2), (3, 0), (0, 4), (1, 5)])
def test_compaction_closed_form_and_brute_force(h, t):
    lens = [h + t, h + t + 1, 19, 64]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    src = RNG.integers(0, 255, size=(cu[-1], 48), dtype=np.uint8)
    res = O.compact_registers(src, cu, h, t)
    r = h + t
    idx, pos = [], []
    for s, n in enumerate(lens):  # brute force: walk every token, keep it if it is a register
        for p in range(n):
            if p < h or p >= n - t:
                idx.append(cu[s] + p)
                pos.append(p)
    np.testing.assert_array_equal(res["idx"], idx)
    np.testing.assert_array_equal(res["pos"], pos)
    np.testing.assert_array_equal(res["cu"], np.arange(len(lens) + 1) * r)
    np.testing.assert_array_equal(res["dst"], src[idx])
    assert np.all(np.diff(res["idx"]) > 0)
    # closed form
    for s, n in enumerate(lens):
        for m in range(r):
            want = cu[s] + (m if m < h else n - t + (m - h))
            assert res["idx"][s * r + m] == want


def test_compaction_without_prompt_is_identity_and_rejects_short_sequences():
    cu = np.array([0, 4, 8], dtype=np.int32)
    src = RNG.integers(0, 255, size=(8, 16), dtype=np.uint8)
    res = O.compact_registers(src, cu, 2, 2)
    np.testing.assert_array_equal(res["idx"], np.arange(8))
    np.testing.assert_array_equal(res["dst"], src)
    with pytest.raises(ValueError):
        O.compact_registers(src, cu, 3, 2)
    with pytest.raises(ValueError):
        O.compact_registers(src, cu, 0, 0)


# ----------------------------------------------------------------------------------------------
# the two definitions of the post-split layers agree (training rule of Section 3.2)
# ----------------------------------------------------------------------------------------------
def test_compacted_layers_equal_full_attention_under_register_key_mask():
    h, t = 3, 2
    lens = [h + t + 20, h + t + 7, h + t]
    q, k, v, cu = rand_batch(lens, 4, 2, 32)
    comp = O.compact_registers(None, cu, h, t)
    idx, pos, cu_c = comp["idx"], comp["pos"], comp["cu"]
    got = O.prefill_attn(q[idx], k[idx], v[idx], cu_c, positions=pos)["out"]
    for s, n in enumerate(lens):
        sl = slice(cu[s], cu[s + 1])
        is_reg = np.zeros(n, dtype=bool)
        is_reg[:h] = True
        is_reg[n - t:] = True
        mask = np.tril(np.ones((n, n), dtype=bool)) & is_reg[None, :]
        # rows of prompt tokens see at least the prefix registers, so no row is empty (h > 0)
        qr, kr = rope_complex(q[sl], np.arange(n), 10000.0), rope_complex(k[sl], np.arange(n), 10000.0)
        ref = dense_masked_attention(qr, kr, v[sl], mask, 2)[is_reg]
        np.testing.assert_allclose(got[cu_c[s]:cu_c[s + 1]], ref, atol=1e-12)


# ----------------------------------------------------------------------------------------------
# decode (Eq. 4)
# ----------------------------------------------------------------------------------------------
def test_decode_step_equals_last_row_of_extended_prefill():
    hq, hkv, d, G = 4, 2, 32, 3
    lens = [9, 14]
    q, k, v, cu = rand_batch(lens, hq, hkv, d)
    pre = O.prefill_attn(q, k, v, cu)
    S = 2
    gen_k = np.zeros((S, G, hkv, d))
    gen_v = np.zeros((S, G, hkv, d))
    dq = RNG.standard_normal((G, S, hq, d))
    dk = RNG.standard_normal((G, S, hkv, d))
    dv = RNG.standard_normal((G, S, hkv, d))
    for g in range(G):
        q_pos = np.array(lens) + g
        res = O.decode_attn(dq[g], dk[g], dv[g], q_pos, pre["k_rot"], v, cu, None, gen_k, gen_v, np.full(S, g))
        assert np.abs(res["rowsum"] - 1).max() < 1e-12
        for s in range(S):  # prefill over the sequence extended by the g+1 generated tokens
            sl = slice(cu[s], cu[s + 1])
            eq = np.concatenate([q[sl], dq[: g + 1, s]])
            ek = np.concatenate([k[sl], dk[: g + 1, s]])
            ev = np.concatenate([v[sl], dv[: g + 1, s]])
            ext = O.prefill_attn(eq, ek, ev, np.array([0, lens[s] + g + 1]))
            np.testing.assert_allclose(res["out"][s], ext["out"][-1], atol=1e-12)
            np.testing.assert_allclose(res["lse"][s], ext["lse"][-1], atol=1e-12)
            np.testing.assert_allclose(gen_k[s, g], ext["k_rot"][-1], atol=1e-13)


def test_decode_on_compacted_cache_equals_masked_full_attention():
    """Layers >= k while decoding: keys are [prefix; suffix; generated] (Section 3.2, decoding bullet)."""
    h, t, hq, hkv, d = 2, 2, 2, 1, 16
    n = 30
    q, k, v, cu = rand_batch([n], hq, hkv, d)
    comp = O.compact_registers(None, cu, h, t)
    pre = O.prefill_attn(q[comp["idx"]], k[comp["idx"]], v[comp["idx"]], comp["cu"], positions=comp["pos"])
    dq, dk, dv = (RNG.standard_normal((1, hq, d)), RNG.standard_normal((1, hkv, d)), RNG.standard_normal((1, hkv, d)))
    gen_k, gen_v = np.zeros((1, 1, hkv, d)), np.zeros((1, 1, hkv, d))
    res = O.decode_attn(dq, dk, dv, [n], pre["k_rot"], v[comp["idx"]], comp["cu"], None, gen_k, gen_v, [0])
    # dense reference over all n+1 tokens with the prompt keys masked out
    aq = rope_complex(np.concatenate([q, dq]), np.arange(n + 1), 10000.0)
    ak = rope_complex(np.concatenate([k, dk]), np.arange(n + 1), 10000.0)
    av = np.concatenate([v, dv])
    allowed = np.zeros(n + 1, dtype=bool)
    allowed[:h] = allowed[n - t:] = True
    mask = np.tril(np.ones((n + 1, n + 1), dtype=bool)) & allowed[None, :]
    ref = dense_masked_attention(aq, ak, av, mask, hq // hkv)[-1]
    np.testing.assert_allclose(res["out"][0], ref, atol=1e-12)


def test_beams_sharing_a_cache_equal_replicated_caches():
    hq, hkv, d, W = 2, 2, 16, 3
    lens = [6, 11]
    _, k, v, cu = rand_batch(lens, hq, hkv, d)
    S = len(lens) * W
    s2s = [u // W for u in range(S)]
    dq, dk, dv = (RNG.standard_normal((S, hq, d)), RNG.standard_normal((S, hkv, d)), RNG.standard_normal((S, hkv, d)))
    q_pos = [lens[s] for s in s2s]
    gk, gv = np.zeros((S, 2, hkv, d)), np.zeros((S, 2, hkv, d))
    shared = O.decode_attn(dq, dk, dv, q_pos, k, v, cu, s2s, gk, gv, np.zeros(S))
    # replicate: every stream gets a private copy of its sequence's cache
    rk = np.concatenate([k[cu[s]:cu[s + 1]] for s in s2s])
    rv = np.concatenate([v[cu[s]:cu[s + 1]] for s in s2s])
    rcu = np.concatenate([[0], np.cumsum([lens[s] for s in s2s])])
    gk2, gv2 = np.zeros((S, 2, hkv, d)), np.zeros((S, 2, hkv, d))
    rep = O.decode_attn(dq, dk, dv, q_pos, rk, rv, rcu, None, gk2, gv2, np.zeros(S))
    np.testing.assert_array_equal(shared["out"], rep["out"])


# ----------------------------------------------------------------------------------------------
# whole path
# ----------------------------------------------------------------------------------------------
def _tiny_inputs(N, k, h, t, lens_hist, hq, hkv, d, G, W=1):
    lens = [h + L + t for L in lens_hist]
    T = sum(lens)
    cu = [0] + list(np.cumsum(lens))
    S = len(lens) * W
    tn = lambda *shape: torch.from_numpy(RNG.standard_normal(shape)).to(torch.float32)
    return dict(n_layers=N, split_k=k, n_head_reg=h, n_tail_reg=t, cu_seqlens=cu,
                q=[tn(T, hq, d) for _ in range(N)], k=[tn(T, hkv, d) for _ in range(N)],
                v=[tn(T, hkv, d) for _ in range(N)], x=tn(T, hq * d),
                dq=[[tn(S, hq, d) for _ in range(N)] for _ in range(G)],
                dk=[[tn(S, hkv, d) for _ in range(N)] for _ in range(G)],
                dv=[[tn(S, hkv, d) for _ in range(N)] for _ in range(G)],
                stream_to_seq=[u // W for u in range(S)])


def test_pipeline_with_split_at_last_layer_is_vanilla_attention():
    """k = N: no layer is register-only, so every prefill output is plain causal attention (library routine)."""
    inp = _tiny_inputs(3, 3, 2, 2, [10, 5], 2, 2, 16, 1)
    out = OP.run(**inp, rope_base=0.0)
    cu = inp["cu_seqlens"]
    for l in range(3):
        for s in range(2):
            sl = slice(cu[s], cu[s + 1])
            tq, tk, tv = (inp[n][l][sl].double().permute(1, 0, 2)[None] for n in ("q", "k", "v"))
            ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2)
            np.testing.assert_allclose(out["prefill_out"][l][sl], ref.numpy(), atol=1e-12)
        assert out["k_cache"][l].shape[0] == cu[-1]


def test_pipeline_shapes_cache_sizes_and_gather_bytes():
    N, k, h, t, G = 4, 2, 2, 1, 2
    inp = _tiny_inputs(N, k, h, t, [12, 0, 7], 2, 1, 16, G, W=2)
    out = OP.run(**inp)
    r, B = h + t, 3
    lens = np.diff(inp["cu_seqlens"])
    for l in range(N):
        rows = inp["cu_seqlens"][-1] if l < k else B * r
        assert out["k_cache"][l].shape[0] == rows and out["prefill_out"][l].shape[0] == rows
    # cache accounting: k full layers + (N-k) register layers + generated tokens in every layer
    for s in range(B):
        held = sum((lens[s] if l < k else r) + G for l in range(N))
        assert out["cache_entries"][s] == held
    # gathered tensors are byte-identical to fancy indexing
    assert torch.equal(out["x_c"], inp["x"][out["idx"]])
    for l in range(k, N):
        assert torch.equal(out["k_c"][l], inp["k"][l][out["idx"]])
    assert len(out["decode_out"]) == G and out["decode_out"][0][0].shape == (6, 2, 16)


# ----------------------------------------------------------------------------------------------
# accounting (Section 3.3, Appendix A.2)
# ----------------------------------------------------------------------------------------------
def _golden():
    vals = {}
    with open(os.path.join(GOLDEN, "efficiency_example.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                key, val = line.split()
                vals[key] = float(val)
    return vals


def test_efficiency_example_printed_by_the_paper():
    g = _golden()
    N, k, L, r = int(g["N"]), int(g["k"]), g["L"], g["r"]
    gc = O.gamma_cache(N, k, L, r)
    assert abs(gc - (N - k) * (L - r) / (N * L)) < 1e-15          # second form printed in the paper
    assert round(100 * gc) == g["cache_reduction_percent"]
    assert N / k == g["speedup"]
    # N_KV per head: k L + (N-k) r, and its ratio to N L
    assert O.cache_entries(N, k, int(L), int(r)) == 8 * 512 + 24 * 2
    assert abs(O.cache_entries(N, k, int(L), int(r)) / (N * L) - (1 - gc)) < 1e-15
    # Gamma_attn ~ k/N for r << L, and the factored form of the per-layer FLOPs
    ga = O.gamma_attn(N, k, L, r, g["n_h"], g["d_a"], g["d_h"], g["d_f"])
    assert abs(ga - k / N) < 3e-3 and ga > k / N
    fl = O.flops_layer(L, g["n_h"], g["d_a"], g["d_h"], g["d_f"])
    assert fl == 4 * L * (g["n_h"] * g["d_a"] * (2 * g["d_h"] + L) + g["d_h"] * g["d_f"])


def test_causal_flop_count():
    # one sequence of length m: 4 d Hq m(m+1)/2
    assert O.causal_attn_flops([100, 132], 4, 64) == 4 * 64 * 4 * (100 * 101 // 2 + 132 * 133 // 2)


# ----------------------------------------------------------------------------------------------
# attention-score statistics (Appendix: Sparsity, Sink_head, Sink_tail)
# ----------------------------------------------------------------------------------------------
def test_attention_statistics_closed_forms():
    """Uniform rows (K = 0): p_j = 1/n, so Sparsity = [1/n > 0.05], Sink_head = min(3, n)/n, Sink_tail = min(4, n)/n
    (T_t = n - 3 makes the tail window four keys wide, as the formula is printed).  Two-level rows: one key with score
    c, all others 0, so p* = e^c / (e^c + n - 1) and the rest share 1 - p*."""
    n, d = 40, 16
    q = RNG.standard_normal((n, 2, d))
    st = O.attn_stats(q, np.zeros((n, 1, d)), [0, n])
    for i in range(n):
        m = i + 1
        np.testing.assert_allclose(st[i, :, 0], 1.0 if 1.0 / m > 0.05 else 0.0)
        np.testing.assert_allclose(st[i, :, 1], min(3, m) / m, rtol=1e-12)
        np.testing.assert_allclose(st[i, :, 2], min(4, m) / m, rtol=1e-12)
    assert st[18, 0, 0] == 1.0 and st[19, 0, 0] == 0.0          # 1/19 > 0.05 >= 1/20: the comparison is strict
    # two-level: without rotation, q = sqrt(d) e_0 scaled by c and key j* = e_0 give score c at j*, 0 elsewhere
    c, jstar = 4.0, 30
    q = np.zeros((n, 1, d)); q[:, 0, 0] = c * np.sqrt(d)
    k = np.zeros((n, 1, d)); k[jstar, 0, 0] = 1.0
    st = O.attn_stats(q, k, [0, n], rope_base=0.0)
    i = n - 1
    pstar = np.exp(c) / (np.exp(c) + n - 1)
    rest = (1 - pstar) / (n - 1)
    assert rest < 0.05 < pstar
    np.testing.assert_allclose(st[i, 0], [1.0 / n, 3 * rest, 4 * rest], rtol=1e-12)          # j* = 31st key: in neither window
    st2 = O.attn_stats(q, np.roll(k, n - 2 - jstar, axis=0), [0, n], rope_base=0.0)            # j* -> the (n-1)th key
    np.testing.assert_allclose(st2[i, 0], [1.0 / n, 3 * rest, pstar + 3 * rest], rtol=1e-12)
    st3 = O.attn_stats(q, np.roll(k, 1 - jstar, axis=0), [0, n], rope_base=0.0)                # j* -> the 2nd key
    np.testing.assert_allclose(st3[i, 0], [1.0 / n, pstar + 2 * rest, 4 * rest], rtol=1e-12)
    # other thresholds and windows
    st4 = O.attn_stats(q, k, [0, n], rope_base=0.0, epsilon=rest / 2, t_head=0, tail_back=n)
    np.testing.assert_allclose(st4[i, 0], [1.0, 0.0, 1.0], rtol=1e-12)


def test_attention_statistics_follow_the_probabilities_of_the_attention_oracle():
    """With rotation, grouped heads and a ragged batch: the statistics are those of the probabilities the (separately
    pinned) attention oracle materialises; and the head map and the explicit scale reach this function as well."""
    lens = [37, 9]
    q, k, v, cu = rand_batch(lens, 4, 2, 32)
    q *= 3.0
    st = O.attn_stats(q, k, cu, scale=0.3)
    for s in range(2):
        for a in range(4):
            p = O.prefill_attn(q, k, v, cu, scale=0.3, want_probs=(s, a))["probs"]
            for i in range(lens[s]):
                m = i + 1
                row = p[i, :m]
                want = [np.mean(row > 0.05), row[:3].sum(), row[max(m - 4, 0):].sum()]
                np.testing.assert_allclose(st[cu[s] + i, a], want, rtol=0, atol=1e-12)
    swapped = O.attn_stats(q, k, cu, q_to_kv=[1, 1, 0, 0], scale=0.3)
    assert np.abs(swapped - st).max() > 1e-3


# ----------------------------------------------------------------------------------------------
# beam search selection (Appendix, implementation details: beam size 20)
# ----------------------------------------------------------------------------------------------
def test_beam_topk_equals_a_stable_sort_and_breaks_ties_by_index():
    batch, beams, vocab = 3, 5, 37
    lp = RNG.standard_normal((batch * beams, vocab)).astype(np.float32)
    lp[2, 5] = lp[7, 30] = lp[7, 31] = 9.0                      # ties at the top, inside and across beams
    lp[11] = -np.inf                                            # a dead beam
    lp[4, 3] = np.nan                                           # never wins
    bs = RNG.standard_normal(batch * beams).astype(np.float32)
    res = O.beam_topk(bs, lp, batch, beams, vocab)
    cand = (lp + bs[:, None]).astype(np.float32).reshape(batch, beams * vocab)   # the fp32 sum
    cand = np.where(np.isnan(cand), -np.inf, cand)
    for b in range(batch):
        order = np.argsort(-cand[b], kind="stable")[:beams]     # library routine: descending, first of equals first
        np.testing.assert_array_equal(res["parent"][b * beams:(b + 1) * beams], b * beams + order // vocab)
        np.testing.assert_array_equal(res["token"][b * beams:(b + 1) * beams], order % vocab)
        np.testing.assert_array_equal(res["score"][b * beams:(b + 1) * beams], cand[b][order])
    # worked by hand: two beams, three tokens
    r = O.beam_topk([0.0, -1.0], [[0.1, 0.5, 0.5], [2.0, 0.1, 1.5]], 1, 2, 3)
    assert r["parent"].tolist() == [1, 0] and r["token"].tolist() == [0, 1] and r["score"].tolist() == [1.0, 0.5]
    # fewer candidates than beams: the rest is empty
    r = O.beam_topk(None, [[0.3], [0.1], [0.2]], 1, 3, 1)
    assert r["parent"].tolist() == [0, 2, 1] and r["token"].tolist() == [0, 0, 0]


# ----------------------------------------------------------------------------------------------
# projections (Appendix A.2)
# ----------------------------------------------------------------------------------------------
def test_qkv_projection_with_rotation():
    rows, dm, hq, hkv, d = 23, 48, 4, 2, 16
    x, w = RNG.standard_normal((rows, dm)), RNG.standard_normal((dm, (hq + 2 * hkv) * d))
    pos = RNG.integers(0, 5000, size=rows)
    res = O.qkv_project(x, w, hq, hkv, d, pos)
    # library matmul in torch + the complex-multiplication form of the rotation
    y = (torch.from_numpy(x) @ torch.from_numpy(w)).numpy()
    np.testing.assert_allclose(res["q"], rope_complex(y[:, : hq * d].reshape(rows, hq, d), pos, 10000.0), rtol=0, atol=1e-9)
    np.testing.assert_allclose(res["k"], rope_complex(y[:, hq * d: (hq + hkv) * d].reshape(rows, hkv, d), pos, 10000.0),
                               rtol=0, atol=1e-9)
    np.testing.assert_allclose(res["v"], y[:, (hq + hkv) * d:].reshape(rows, hkv, d), rtol=0, atol=1e-12)   # V is not rotated
    # position 0 and rope_base 0: the plain product; a selector matrix: rotated copies of x's columns
    plain = O.qkv_project(x, w, hq, hkv, d, np.zeros(rows, dtype=np.int32))
    np.testing.assert_allclose(plain["q"].reshape(rows, -1), y[:, : hq * d], rtol=0, atol=1e-12)
    np.testing.assert_allclose(O.qkv_project(x, w, hq, hkv, d, pos, rope_base=0.0)["k"], plain["k"], rtol=0, atol=1e-12)
    sel = np.zeros((dm, (hq + 2 * hkv) * d)); sel[:16, hq * d: hq * d + 16] = np.eye(16)   # K head 0 = x[:, :16]
    np.testing.assert_allclose(O.qkv_project(x, sel, hq, hkv, d, pos)["k"][:, 0], O.rope(x[:, None, :16], pos)[:, 0], atol=1e-12)
    # feeding the attention oracle rotated projections with its own rotation off = feeding it the raw projections
    cu = [0, 10, 23]
    p2 = np.concatenate([np.arange(10), np.arange(13)])
    raw = O.qkv_project(x, w, hq, hkv, d, p2, rope_base=0.0)
    rot = O.qkv_project(x, w, hq, hkv, d, p2)
    a = O.prefill_attn(raw["q"], raw["k"], raw["v"], cu)["out"]
    b = O.prefill_attn(rot["q"], rot["k"], rot["v"], cu, rope_base=0.0)["out"]
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-10)


def test_linear_and_silu_equal_the_library_routines():
    x, w = RNG.standard_normal((9, 32)), RNG.standard_normal((32, 24))
    np.testing.assert_allclose(O.linear(x, w), torch.nn.functional.linear(torch.from_numpy(x), torch.from_numpy(w).T).numpy(),
                               rtol=0, atol=1e-12)
    want = torch.nn.functional.silu(torch.from_numpy(x) @ torch.from_numpy(w)).numpy()
    np.testing.assert_allclose(O.linear(x, w, 1), want, rtol=0, atol=1e-12)


# ----------------------------------------------------------------------------------------------
# backward of the attention (Section 3.2, Training)
# ----------------------------------------------------------------------------------------------
def test_attention_backward_equals_autograd_of_the_library_attention():
    lens, hq, hkv, d = [1, 17, 40], 6, 2, 16
    q, k, v, cu = rand_batch(lens, hq, hkv, d)
    g = RNG.standard_normal(q.shape)
    res = O.attn_backward(q, k, v, g, cu, scale=0.3)
    for s in range(len(lens)):
        sl = slice(cu[s], cu[s + 1])
        tq = torch.from_numpy(q[sl]).clone().requires_grad_(True)
        tk = torch.from_numpy(k[sl]).clone().requires_grad_(True)
        tv = torch.from_numpy(v[sl]).clone().requires_grad_(True)
        rep = lambda t: t.repeat_interleave(hq // hkv, dim=1).permute(1, 0, 2)[None]
        o = torch.nn.functional.scaled_dot_product_attention(tq.permute(1, 0, 2)[None], rep(tk), rep(tv), is_causal=True, scale=0.3)
        o.backward(torch.from_numpy(g[sl]).permute(1, 0, 2)[None])
        np.testing.assert_allclose(res["dq"][sl], tq.grad.numpy(), rtol=0, atol=1e-11)
        np.testing.assert_allclose(res["dk"][sl], tk.grad.numpy(), rtol=0, atol=1e-11)     # summed over the group's heads
        np.testing.assert_allclose(res["dv"][sl], tv.grad.numpy(), rtol=0, atol=1e-11)
    # a central difference of the forward oracle through one element of each input
    f = lambda qq, kk, vv: float((O.prefill_attn(qq, kk, vv, cu, scale=0.3, rope_base=0.0)["out"] * g).sum())
    for name, arr, grad, at in (("q", q, res["dq"], (30, 4, 3)), ("k", k, res["dk"], (20, 1, 7)), ("v", v, res["dv"], (5, 0, 2))):
        hi, lo = arr.copy(), arr.copy()
        hi[at] += 1e-5
        lo[at] -= 1e-5
        args = {"q": (hi, k, v), "k": (q, hi, v), "v": (q, k, hi)}[name], {"q": (lo, k, v), "k": (q, lo, v), "v": (q, k, lo)}[name]
        assert abs((f(*args[0]) - f(*args[1])) / 2e-5 - grad[at]) < 1e-6, name
    # the explicit head map reaches the backward as well
    assert np.abs(O.attn_backward(q, k, v, g, cu, q_to_kv=[1, 1, 0, 0, 1, 0])["dk"] - O.attn_backward(q, k, v, g, cu)["dk"]).max() > 1e-3
