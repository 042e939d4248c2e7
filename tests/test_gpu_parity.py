"""Parity of the HIP path (through the C ABI) with the fp64 CPU oracle, on the same seeded inputs.

Bars: bit-exact for compaction (indices and gathered bytes); max-abs <= 1e-4 for fp32 attention outputs;
||O_gpu - O_ref||_F / ||O_ref||_F <= 2e-2 for bf16 attention outputs.
"""
import numpy as np
import pytest
import torch

from oracle import earn_oracle as O
from oracle import pipeline as OP
from paper_2507_00715_amd import workloads as W
from parity import BF16_REL, F32_ATOL, check_attn, rel_fro, vector_bar

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _B():
    from paper_2507_00715_amd import binding
    binding.lib()
    return binding


def make_cfg(dtype, hq, hkv, d, h=2, t=2, N=1, k=1, G=1, W_=1, outlier=0.0):
    return W.Config("test", 77, "f32" if dtype == torch.float32 else "bf16", 0, ("fixed", 0), h, t, N, k, hq, hkv, d, G,
                    beams=W_, outlier_prob=outlier)


def make_workload(cfg, hist):
    return W.Workload(cfg.replace(batch=len(hist)), history_lengths=hist)


# --------------------------------------------------------------------------------------------------
def test_generator_is_bit_identical_on_cpu_and_gpu():
    w = W.Workload(W.CONFIGS["small_gqa"])
    for which in ("q", "k", "v", "x"):
        a = w.prefill_tensor(which, 2, seqs=[0, 7])
        b = w.prefill_tensor(which, 2, device=DEV, seqs=[0, 7])
        assert torch.equal(a, b.cpu())
    w3 = W.Workload(W.CONFIGS["mid_mha"])
    assert torch.equal(w3.prefill_tensor("k", 1, seqs=[1]), w3.prefill_tensor("k", 1, device=DEV, seqs=[1]).cpu())
    assert torch.equal(w.decode_tensor("q", 3, 5), w.decode_tensor("q", 3, 5, device=DEV).cpu())


# --------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("h,t,lens", [(2, 2, [100, 132]), (8, 8, [16, 17, 300, 16, 511]), (3, 0, [3, 40, 9]),
                                      (0, 5, [5, 6, 77]), (32, 32, [64, 8256, 100])])
def test_compaction_is_bit_exact(h, t, lens):
    B = _B()
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T, batch, r = int(cu[-1]), len(lens), h + t
    g = torch.Generator().manual_seed(T)
    srcs = [torch.randint(-2**15, 2**15 - 1, (T, 4, 64), dtype=torch.int16, generator=g),      # a bf16 K/V row
            torch.randint(0, 255, (T, 16), dtype=torch.uint8, generator=g),                      # smallest legal row
            torch.randint(-2**31, 2**31 - 1, (T, 1028), dtype=torch.int32, generator=g)]         # 4112-byte rows
    d_src = [s.to(DEV) for s in srcs]
    d_dst = [torch.zeros((batch * r,) + tuple(s.shape[1:]), dtype=s.dtype, device=DEV) for s in srcs]
    d_cu = torch.from_numpy(cu).to(DEV)
    idx = torch.full((batch * r,), -1, dtype=torch.int32, device=DEV)
    pos = torch.full((batch * r,), -1, dtype=torch.int32, device=DEV)
    cu_c = torch.full((batch + 1,), -1, dtype=torch.int32, device=DEV)
    B.earn_compact_registers(d_src, d_dst, d_cu, batch, h, t, idx, pos, cu_c)
    torch.cuda.synchronize()
    ref = O.compact_registers(None, cu, h, t)
    np.testing.assert_array_equal(idx.cpu().numpy(), ref["idx"])
    np.testing.assert_array_equal(pos.cpu().numpy(), ref["pos"])
    np.testing.assert_array_equal(cu_c.cpu().numpy(), ref["cu"])
    for s, dd in zip(srcs, d_dst):
        want = O.compact_registers(s.numpy(), cu, h, t)["dst"]
        assert np.array_equal(dd.cpu().numpy(), want)
    # index outputs only
    idx2 = torch.empty_like(idx)
    B.earn_compact_registers([], [], d_cu, batch, h, t, idx2, None, None)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(idx2.cpu().numpy(), ref["idx"])


# --------------------------------------------------------------------------------------------------
def run_prefill(B, w, layer, positions=None, coords=None, cu=None, want_lse=True, k_rot=True):
    cfg = w.cfg
    q = w.prefill_tensor("q", layer, coords=coords)
    k = w.prefill_tensor("k", layer, coords=coords)
    v = w.prefill_tensor("v", layer, coords=coords)
    cu = w.cu_seqlens if cu is None else cu
    T, batch = q.shape[0], len(cu) - 1
    max_len = int(np.diff(cu).max())
    desc = B.make_desc(cfg.torch_dtype, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, 0.0, cfg.rope_base)
    dq, dk, dv = q.to(DEV), k.to(DEV), v.to(DEV)
    out = torch.full_like(dq, float("nan"))
    krot = torch.full_like(dk, float("nan")) if k_rot else None
    lse = torch.full((T, cfg.n_q_heads), float("nan"), device=DEV) if want_lse else None
    ws_bytes = B.earn_prefill_workspace_bytes(desc, batch, T, max_len, k_rot)
    ws = torch.empty(max(ws_bytes, 1), dtype=torch.uint8, device=DEV)
    dcu = torch.tensor(list(cu), dtype=torch.int32, device=DEV)
    dpos = None if positions is None else torch.tensor(list(positions), dtype=torch.int32, device=DEV)
    B.earn_prefill_attn(desc, dq, dk, dv, dcu, dpos, batch, T, max_len, out, krot, lse, ws)
    torch.cuda.synchronize()
    ref = O.prefill_attn(W.to_f64(q), W.to_f64(k), W.to_f64(v), cu, positions, rope_base=cfg.rope_base)
    return out, krot, lse, ref


PREFILL_CASES = [
    # dtype, hq, hkv, d, history lengths (sequence length = history + 4)
    (torch.float32, 4, 4, 64, [96, 128]),
    (torch.float32, 6, 2, 128, [0, 1, 61, 130]),
    (torch.bfloat16, 14, 2, 64, [0, 1, 59, 60, 61, 252, 253, 300, 521]),
    (torch.bfloat16, 4, 4, 128, [27, 256, 700]),
    (torch.bfloat16, 8, 2, 128, [1100, 60, 508]),
]


@pytest.mark.parametrize("dtype,hq,hkv,d,hist", PREFILL_CASES)
def test_prefill_matches_oracle(dtype, hq, hkv, d, hist):
    B = _B()
    w = make_workload(make_cfg(dtype, hq, hkv, d), hist)
    out, krot, lse, ref = run_prefill(B, w, 0)
    check_attn(out, ref["out"], dtype, "out")
    check_attn(krot, ref["k_rot"], dtype, "k_rot")
    lse_err = np.abs(lse.cpu().double().numpy() - ref["lse"]).max()
    assert lse_err < (1e-4 if dtype == torch.float32 else 5e-2), f"lse err {lse_err}"
    # without k_rot_out the rotated keys go to the workspace: same result
    out2, _, _, _ = run_prefill(B, w, 0, want_lse=False, k_rot=False)
    assert torch.equal(out, out2)


@pytest.mark.parametrize("dtype,hq,hkv,d", [(torch.float32, 4, 4, 64), (torch.bfloat16, 14, 2, 64),
                                            (torch.bfloat16, 32, 8, 128)])
def test_prefill_on_compacted_rows_with_original_positions(dtype, hq, hkv, d):
    B = _B()
    h, t = 8, 8
    w = make_workload(make_cfg(dtype, hq, hkv, d, h=h, t=t), [300, 0, 4000, 77])
    comp = O.compact_registers(None, np.asarray(w.cu_seqlens, dtype=np.int32), h, t)
    seq = torch.repeat_interleave(torch.arange(w.cfg.batch), h + t)
    coords = (seq, torch.from_numpy(comp["pos"]).long())
    out, krot, _, ref = run_prefill(B, w, 1, positions=comp["pos"], coords=coords, cu=comp["cu"])
    check_attn(out, ref["out"], dtype, "out")
    check_attn(krot, ref["k_rot"], dtype, "k_rot")
    # negative control: positions 0..r-1 instead of the original ones give a different answer
    ref_renum = O.prefill_attn(W.to_f64(w.prefill_tensor("q", 1, coords=coords)),
                               W.to_f64(w.prefill_tensor("k", 1, coords=coords)),
                               W.to_f64(w.prefill_tensor("v", 1, coords=coords)), comp["cu"], None)
    assert rel_fro(out.cpu().double().numpy(), ref_renum["out"]) > 5e-2


def test_prefill_with_outlier_keys():
    """5 % of key rows scaled x8 (attention-sink-like outliers) keep the bf16 path inside the tolerance."""
    B = _B()
    w = make_workload(make_cfg(torch.bfloat16, 4, 4, 128, outlier=0.05), [900, 333])
    out, _, _, ref = run_prefill(B, w, 0)
    check_attn(out, ref["out"], torch.bfloat16, "out", vector_bar(w.cfg.outlier_scale))


def test_prefill_without_rope():
    B = _B()
    w = make_workload(make_cfg(torch.bfloat16, 4, 2, 64).replace(rope_base=0.0), [200])
    out, krot, _, ref = run_prefill(B, w, 0)
    check_attn(out, ref["out"], torch.bfloat16)
    assert torch.equal(krot.cpu(), w.prefill_tensor("k", 0))


# --------------------------------------------------------------------------------------------------
DECODE_CASES = [
    # dtype, hq, hkv, d, shared lengths, beams, gen_len per stream pattern, gen_cap
    (torch.float32, 4, 4, 64, [100, 132], 1, [0, 3], 4),
    (torch.float32, 6, 2, 128, [5, 0, 70], 2, [0, 1, 2, 0, 1, 2], 3),
    (torch.bfloat16, 14, 2, 64, [16, 16, 300, 524], 1, [0, 15, 7, 1], 16),
    (torch.bfloat16, 32, 32, 128, [32, 2059, 700], 1, [2, 0, 7], 8),
    (torch.bfloat16, 32, 8, 128, [64, 8256], 3, [0, 1, 2, 3, 4, 7], 8),
    (torch.bfloat16, 12, 2, 128, [16, 1038, 81], 1, [3, 0, 1], 4),
    # beams: 4 heads x 20 beams = 80 query rows per cache (more than one 64-row pass), ragged last tile, empty cache
    (torch.bfloat16, 32, 8, 128, [64, 2100, 0], 20, [i % 5 for i in range(60)], 5),
    (torch.bfloat16, 14, 2, 64, [300, 16, 1000], 6, [i % 3 for i in range(18)], 3),
    (torch.bfloat16, 8, 8, 64, [33, 700], 4, [0, 1, 2, 3, 3, 2, 1, 0], 4),
    # long generated caches of very different lengths: the generated rows span several key tiles
    (torch.bfloat16, 8, 2, 128, [500, 129], 2, [199, 70, 0, 130], 200),
    (torch.bfloat16, 4, 2, 64, [256], 3, [64, 63, 0], 65),
    # enough (sequence, kv head) pairs to fill the GPU without splitting key ranges: final outputs without a merge pass
    (torch.bfloat16, 16, 8, 64, [130 + 7 * (i % 5) for i in range(32)], 1, [i % 3 for i in range(32)], 3),
]


@pytest.mark.parametrize("dtype,hq,hkv,d,slens,beams,glens,gen_cap", DECODE_CASES)
def test_decode_matches_oracle(dtype, hq, hkv, d, slens, beams, glens, gen_cap):
    B = _B()
    gtor = torch.Generator().manual_seed(sum(slens) + hq)
    rnd = lambda *shape: torch.randn(*shape, generator=gtor).to(dtype)
    batch, S = len(slens), len(slens) * beams
    cu = np.concatenate([[0], np.cumsum(slens)]).astype(np.int32)
    s2s = [u // beams for u in range(S)]
    sk, sv = rnd(int(cu[-1]), hkv, d), rnd(int(cu[-1]), hkv, d)
    q, kn, vn = rnd(S, hq, d), rnd(S, hkv, d), rnd(S, hkv, d)
    gk, gv = rnd(S, gen_cap, hkv, d), rnd(S, gen_cap, hkv, d)
    q_pos = [slens[s2s[u]] + glens[u] + 5 for u in range(S)]
    desc = B.make_desc(dtype, hq, hkv, d)
    dev = lambda x: x.to(DEV)
    d_gk, d_gv = dev(gk), dev(gv)
    out = torch.full((S, hq, d), float("nan"), dtype=dtype, device=DEV)
    ws = torch.empty(max(B.earn_decode_workspace_bytes(desc, S, batch, max(slens), gen_cap), 1), dtype=torch.uint8,
                     device=DEV)
    i32 = lambda x: torch.tensor(list(x), dtype=torch.int32, device=DEV)
    B.earn_decode_attn(desc, dev(q), dev(kn), dev(vn), i32(q_pos), dev(sk), dev(sv), i32(cu), i32(s2s), d_gk, d_gv,
                       i32(glens), gen_cap, S, batch, max(slens), out, ws)
    torch.cuda.synchronize()
    o_gk, o_gv = W.to_f64(gk), W.to_f64(gv)
    ref = O.decode_attn(W.to_f64(q), W.to_f64(kn), W.to_f64(vn), q_pos, W.to_f64(sk), W.to_f64(sv), cu, s2s, o_gk, o_gv,
                        glens)
    check_attn(out, ref["out"], dtype, "out")
    # cache append: slot gen_len[u] holds the rotated key / the value; every other slot is untouched
    got_gk, got_gv = d_gk.cpu(), d_gv.cpu()
    for u in range(S):
        g = glens[u]
        check_attn(got_gk[u, g], o_gk[u, g], dtype, "gen_k slot")
        assert torch.equal(got_gv[u, g], vn[u])
        keep = [j for j in range(gen_cap) if j != g]
        assert torch.equal(got_gk[u, keep], gk[u, keep]) and torch.equal(got_gv[u, keep], gv[u, keep])


@pytest.mark.parametrize("hq,hkv,d,beams", [(8, 2, 128, 3), (4, 4, 64, 1)])
def test_decode_with_late_outlier_keys(hq, hkv, d, beams):
    """Keys far larger than everything before them, late in the cache and among the generated rows: the running softmax
    reference has to be replaced in the middle of the key list (matrix-core kernel: exact path; vector kernel: rescale)."""
    B = _B()
    dtype, gen_cap = torch.bfloat16, 6
    slens = [900, 200]
    batch, S = len(slens), len(slens) * beams
    s2s = [u // beams for u in range(S)]
    glens = [(u * 2) % gen_cap for u in range(S)]
    gtor = torch.Generator().manual_seed(5 + hq)
    rnd = lambda *shape: torch.randn(*shape, generator=gtor).to(dtype)
    cu = np.concatenate([[0], np.cumsum(slens)]).astype(np.int32)
    sk, sv = rnd(int(cu[-1]), hkv, d), rnd(int(cu[-1]), hkv, d)
    sk[700:720] *= 30.0          # late in sequence 0
    sk[cu[1] + 150] *= 40.0      # one key near the end of sequence 1
    q, kn, vn = rnd(S, hq, d), rnd(S, hkv, d), rnd(S, hkv, d)
    gk, gv = rnd(S, gen_cap, hkv, d), rnd(S, gen_cap, hkv, d)
    gk[0, 0] *= 50.0             # and a generated row
    q_pos = [slens[s2s[u]] + glens[u] for u in range(S)]
    desc = B.make_desc(dtype, hq, hkv, d)
    dev = lambda x: x.to(DEV)
    i32 = lambda x: torch.tensor(list(x), dtype=torch.int32, device=DEV)
    d_gk, d_gv = dev(gk), dev(gv)
    out = torch.full((S, hq, d), float("nan"), dtype=dtype, device=DEV)
    ws = torch.empty(max(B.earn_decode_workspace_bytes(desc, S, batch, max(slens), gen_cap), 1), dtype=torch.uint8, device=DEV)
    B.earn_decode_attn(desc, dev(q), dev(kn), dev(vn), i32(q_pos), dev(sk), dev(sv), i32(cu), i32(s2s), d_gk, d_gv,
                       i32(glens), gen_cap, S, batch, max(slens), out, ws)
    torch.cuda.synchronize()
    o_gk, o_gv = W.to_f64(gk), W.to_f64(gv)
    ref = O.decode_attn(W.to_f64(q), W.to_f64(kn), W.to_f64(vn), q_pos, W.to_f64(sk), W.to_f64(sv), cu, s2s, o_gk, o_gv,
                        glens)
    got = out.cpu().double().numpy()
    assert np.isfinite(got).all()
    check_attn(got, ref["out"], dtype, "out")


def test_decode_with_many_and_unevenly_spread_beams():
    """More query rows per cache than one pass of the matrix-core kernel takes (the passes get workgroups of their own,
    planned from the average beam count), with one sequence holding most of the streams and one holding none."""
    B = _B()
    dtype, hq, hkv, d, gen_cap = torch.bfloat16, 8, 2, 128, 4
    slens = [700, 260, 300]
    s2s = [0] * 45 + [1] * 5          # 180 query rows on sequence 0, 20 on sequence 1, none on sequence 2
    S, batch = len(s2s), len(slens)
    glens = [u % 4 for u in range(S)]
    gtor = torch.Generator().manual_seed(99)
    rnd = lambda *shape: torch.randn(*shape, generator=gtor).to(dtype)
    cu = np.concatenate([[0], np.cumsum(slens)]).astype(np.int32)
    sk, sv = rnd(int(cu[-1]), hkv, d), rnd(int(cu[-1]), hkv, d)
    q, kn, vn = rnd(S, hq, d), rnd(S, hkv, d), rnd(S, hkv, d)
    gk, gv = rnd(S, gen_cap, hkv, d), rnd(S, gen_cap, hkv, d)
    q_pos = [slens[s2s[u]] + glens[u] for u in range(S)]
    desc = B.make_desc(dtype, hq, hkv, d)
    dev = lambda x: x.to(DEV)
    i32 = lambda x: torch.tensor(list(x), dtype=torch.int32, device=DEV)
    d_gk, d_gv = dev(gk), dev(gv)
    out = torch.full((S, hq, d), float("nan"), dtype=dtype, device=DEV)
    ws = torch.empty(max(B.earn_decode_workspace_bytes(desc, S, batch, max(slens), gen_cap), 1), dtype=torch.uint8, device=DEV)
    B.earn_decode_attn(desc, dev(q), dev(kn), dev(vn), i32(q_pos), dev(sk), dev(sv), i32(cu), i32(s2s), d_gk, d_gv,
                       i32(glens), gen_cap, S, batch, max(slens), out, ws)
    torch.cuda.synchronize()
    o_gk, o_gv = W.to_f64(gk), W.to_f64(gv)
    ref = O.decode_attn(W.to_f64(q), W.to_f64(kn), W.to_f64(vn), q_pos, W.to_f64(sk), W.to_f64(sv), cu, s2s, o_gk, o_gv,
                        glens)
    got = out.cpu().double().numpy()
    assert np.isfinite(got).all()
    check_attn(got, ref["out"], dtype, "out")
    for u in range(S):
        check_attn(d_gk[u, glens[u]], o_gk[u, glens[u]], dtype, "gen_k slot")
        assert torch.equal(d_gv[u, glens[u]].cpu(), vn[u])
        keep = [j for j in range(gen_cap) if j != glens[u]]
        assert torch.equal(d_gk[u, keep].cpu(), gk[u, keep]) and torch.equal(d_gv[u, keep].cpu(), gv[u, keep])


@pytest.mark.parametrize("dtype,hq,hkv,d,slens", [(torch.bfloat16, 8, 2, 128, [300, 129, 1000]),   # matrix-core kernel
                                                   (torch.bfloat16, 4, 4, 64, [300, 16, 70]),        # vector kernel
                                                   (torch.float32, 4, 2, 64, [40, 9])])
def test_decode_without_stream_map(dtype, hq, hkv, d, slens):
    """stream_to_seq = NULL means one stream per sequence, stream u reading sequence u's cache."""
    B = _B()
    gtor = torch.Generator().manual_seed(7 * sum(slens) + hq)
    rnd = lambda *shape: torch.randn(*shape, generator=gtor).to(dtype)
    S = len(slens)
    glens, gen_cap = [u % 3 for u in range(S)], 3
    cu = np.concatenate([[0], np.cumsum(slens)]).astype(np.int32)
    sk, sv = rnd(int(cu[-1]), hkv, d), rnd(int(cu[-1]), hkv, d)
    q, kn, vn = rnd(S, hq, d), rnd(S, hkv, d), rnd(S, hkv, d)
    gk, gv = rnd(S, gen_cap, hkv, d), rnd(S, gen_cap, hkv, d)
    q_pos = [slens[u] + glens[u] for u in range(S)]
    desc = B.make_desc(dtype, hq, hkv, d)
    dev = lambda x: x.to(DEV)
    i32 = lambda x: torch.tensor(list(x), dtype=torch.int32, device=DEV)
    d_gk, d_gv = dev(gk), dev(gv)
    out = torch.full((S, hq, d), float("nan"), dtype=dtype, device=DEV)
    ws = torch.empty(max(B.earn_decode_workspace_bytes(desc, S, S, max(slens), gen_cap), 1), dtype=torch.uint8, device=DEV)
    B.earn_decode_attn(desc, dev(q), dev(kn), dev(vn), i32(q_pos), dev(sk), dev(sv), i32(cu), None, d_gk, d_gv,
                       i32(glens), gen_cap, S, S, max(slens), out, ws)
    torch.cuda.synchronize()
    o_gk, o_gv = W.to_f64(gk), W.to_f64(gv)
    ref = O.decode_attn(W.to_f64(q), W.to_f64(kn), W.to_f64(vn), q_pos, W.to_f64(sk), W.to_f64(sv), cu, list(range(S)),
                        o_gk, o_gv, glens)
    check_attn(out, ref["out"], dtype, "out")
    for u in range(S):
        check_attn(d_gk[u, glens[u]], o_gk[u, glens[u]], dtype, "gen_k slot")
        assert torch.equal(d_gv[u, glens[u]].cpu(), vn[u])


def test_bound_calls_equal_direct_calls():
    """A call marshalled once (binding.BoundCall) enqueues exactly what the direct call does, every time it is called."""
    B = _B()
    dtype, hq, hkv, d, gen_cap = torch.bfloat16, 8, 2, 64, 3
    slens = [200, 40]
    S = batch = len(slens)
    gtor = torch.Generator().manual_seed(11)
    rnd = lambda *shape: torch.randn(*shape, generator=gtor).to(dtype).to(DEV)
    cu = torch.tensor([0, 200, 240], dtype=torch.int32, device=DEV)
    sk, sv, q, kn, vn = rnd(240, hkv, d), rnd(240, hkv, d), rnd(S, hq, d), rnd(S, hkv, d), rnd(S, hkv, d)
    gk0, gv0 = rnd(S, gen_cap, hkv, d), rnd(S, gen_cap, hkv, d)
    glen = torch.tensor([1, 2], dtype=torch.int32, device=DEV)
    qpos = torch.tensor([201, 42], dtype=torch.int32, device=DEV)
    desc = B.make_desc(dtype, hq, hkv, d)
    ws = torch.empty(max(B.earn_decode_workspace_bytes(desc, S, batch, 200, gen_cap), 1), dtype=torch.uint8, device=DEV)
    gk1, gv1, out1 = gk0.clone(), gv0.clone(), torch.empty_like(q)
    B.earn_decode_attn(desc, q, kn, vn, qpos, sk, sv, cu, None, gk1, gv1, glen, gen_cap, S, batch, 200, out1, ws)
    gk2, gv2, out2 = gk0.clone(), gv0.clone(), torch.full_like(q, float("nan"))
    call = B.bind_decode_attn(desc, q, kn, vn, qpos, sk, sv, cu, None, gk2, gv2, glen, gen_cap, S, batch, 200, out2, ws)
    for _ in range(3):
        out2.fill_(float("nan"))
        call()
        torch.cuda.synchronize()
        assert torch.equal(out1, out2) and torch.equal(gk1, gk2) and torch.equal(gv1, gv2)
    # prefill
    T = 240
    qf, out_a, out_b = rnd(T, hq, d), torch.empty(T, hq, d, dtype=dtype, device=DEV), torch.empty(T, hq, d, dtype=dtype, device=DEV)
    kr_a, kr_b = torch.empty_like(sk), torch.empty_like(sk)
    pws = torch.empty(max(B.earn_prefill_workspace_bytes(desc, batch, T, 200, True), 256), dtype=torch.uint8, device=DEV)
    B.earn_prefill_attn(desc, qf, sk, sv, cu, None, batch, T, 200, out_a, kr_a, None, pws)
    B.bind_prefill_attn(desc, qf, sk, sv, cu, None, batch, T, 200, out_b, kr_b, None, pws)()
    torch.cuda.synchronize()
    assert torch.equal(out_a, out_b) and torch.equal(kr_a, kr_b)


# --------------------------------------------------------------------------------------------------
def _pipeline_inputs(w, device):
    cfg = w.cfg
    N, G = cfg.n_layers, cfg.decode_steps
    mk = lambda which: [w.prefill_tensor(which, l, device=device) for l in range(N)]
    dmk = lambda which: [[w.decode_tensor(which, l, g, device=device) for l in range(N)] for g in range(G)]
    return dict(q=mk("q"), k=mk("k"), v=mk("v"), x=w.prefill_tensor("x", 0, device=device), dq=dmk("q"), dk=dmk("k"),
                dv=dmk("v"))


@pytest.mark.parametrize("name,hist", [("tiny_f32", None), ("small_gqa", [256, 300, 512, 0, 64])])
def test_whole_path_matches_oracle(name, hist):
    """Prefill of k full layers, compaction, N-k register layers and G decode steps, layer by layer."""
    _B()
    from paper_2507_00715_amd.pipeline import EarnPath
    cfg = W.CONFIGS[name]
    if hist is not None:
        cfg = cfg.replace(batch=len(hist), n_layers=6, split_k=2, decode_steps=3)
    w = W.Workload(cfg, history_lengths=hist)
    cpu, gpu = _pipeline_inputs(w, "cpu"), _pipeline_inputs(w, DEV)
    ref = OP.run(n_layers=cfg.n_layers, split_k=cfg.split_k, n_head_reg=cfg.n_head_reg, n_tail_reg=cfg.n_tail_reg,
                 cu_seqlens=w.cu_seqlens, stream_to_seq=w.stream_to_seq, rope_base=cfg.rope_base, **cpu)
    path = EarnPath(n_layers=cfg.n_layers, split_k=cfg.split_k, n_head_reg=cfg.n_head_reg, n_tail_reg=cfg.n_tail_reg,
                    n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim, dtype=cfg.torch_dtype,
                    cu_seqlens=w.cu_seqlens, stream_to_seq=w.stream_to_seq, gen_cap=cfg.decode_steps,
                    rope_base=cfg.rope_base, device=DEV)
    path.prefill(gpu["q"], gpu["k"], gpu["v"], gpu["x"])
    torch.cuda.synchronize()
    # compaction: bit-exact indices and gathered bytes
    np.testing.assert_array_equal(path.idx.cpu().numpy(), ref["idx"])
    np.testing.assert_array_equal(path.pos.cpu().numpy(), ref["pos"])
    np.testing.assert_array_equal(path.cu_c.cpu().numpy(), ref["cu_c"])
    assert torch.equal(path.x_c.cpu(), ref["x_c"])
    for l in range(cfg.split_k, cfg.n_layers):
        assert torch.equal(path.q_c[l].cpu(), ref["q_c"][l]) and torch.equal(path.k_c[l].cpu(), ref["k_c"][l])
        assert torch.equal(path.v_c[l].cpu(), ref["v_c"][l])
    for l in range(cfg.n_layers):
        check_attn(path.prefill_out[l], ref["prefill_out"][l], cfg.torch_dtype, f"prefill layer {l}")
        check_attn(path.k_cache[l], ref["k_cache"][l], cfg.torch_dtype, f"k cache layer {l}")
    for g in range(cfg.decode_steps):
        path.decode_step(g, gpu["dq"][g], gpu["dk"][g], gpu["dv"][g])
        torch.cuda.synchronize()
        for l in range(cfg.n_layers):
            check_attn(path.decode_out[l], ref["decode_out"][g][l], cfg.torch_dtype, f"decode step {g} layer {l}")
    # cache accounting: what the path holds equals the closed form k n + (N-k) r (+ generated)
    from paper_2507_00715_amd import binding as B
    for s in range(cfg.batch):
        held = sum(path.k_cache[l].shape[0] // cfg.batch if l >= cfg.split_k else w.seq_lengths[s]
                   for l in range(cfg.n_layers)) + cfg.n_layers * cfg.decode_steps
        assert held == B.earn_cache_entries(cfg.n_layers, cfg.split_k, w.seq_lengths[s], cfg.r, cfg.decode_steps)
        assert held == ref["cache_entries"][s]
