"""The layer-batched entry points (several independent layers in one launch) against the single-layer calls on every
layer and against the fp64 oracle, and earn_decode_step_positions against the position rule written out."""
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


def i32(x):
    return torch.tensor(list(x), dtype=torch.int32, device=DEV)


PREFILL_CASES = [
    (BF, 8, 2, 128, [40, 16, 64], 5, True),     # register-sized sequences, explicit positions
    (BF, 14, 2, 64, [300, 61, 1000], 3, False),  # 128-row workgroups
    (BF, 4, 2, 128, [3300, 1000], 2, False),     # pipelined kernel (sequences long on average)
    (F32, 6, 2, 64, [130, 70], 4, True),         # vector kernel
]


@pytest.mark.parametrize("dtype,hq,hkv,d,lens,n_layers,explicit_pos", PREFILL_CASES)
def test_prefill_layers_equal_single_layer_calls_and_oracle(dtype, hq, hkv, d, lens, n_layers, explicit_pos):
    B = _B()
    T, batch = sum(lens), len(lens)
    g = torch.Generator().manual_seed(T + hq + n_layers)
    rnd = lambda *s: torch.randn(*s, generator=g).to(dtype)
    q, k, v = rnd(n_layers, T, hq, d), rnd(n_layers, T, hkv, d), rnd(n_layers, T, hkv, d)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    pos = None
    if explicit_pos:  # ascending inside each sequence, with gaps (what compacted register rows carry)
        pos = np.concatenate([np.arange(n) * 3 + 7 * (n > 20) * (np.arange(n) >= n // 2) for n in lens]).astype(np.int32)
    desc = B.make_desc(dtype, hq, hkv, d)
    dq, dk, dv = q.to(DEV), k.to(DEV), v.to(DEV)
    dcu = torch.from_numpy(cu).to(DEV)
    dpos = None if pos is None else torch.from_numpy(pos).to(DEV)
    # a stride larger than the layer itself: the stack is a slice of a wider allocation
    out_wide = torch.full((n_layers, T + 3, hq, d), float("nan"), dtype=dtype, device=DEV)
    out = out_wide[:, :T]
    krot = torch.full((n_layers, T, hkv, d), float("nan"), dtype=dtype, device=DEV)
    lse = torch.full((n_layers, T, hq), float("nan"), dtype=torch.float32, device=DEV)
    B.earn_prefill_attn_layers(desc, dq, dk, dv, dcu, dpos, batch, T, max(lens), out, krot, lse)
    torch.cuda.synchronize()
    for l in range(n_layers):
        o1 = torch.empty(T, hq, d, dtype=dtype, device=DEV)
        k1 = torch.empty(T, hkv, d, dtype=dtype, device=DEV)
        l1 = torch.empty(T, hq, dtype=torch.float32, device=DEV)
        B.earn_prefill_attn(desc, dq[l], dk[l], dv[l], dcu, dpos, batch, T, max(lens), o1, k1, l1, None)
        torch.cuda.synchronize()
        assert torch.equal(out[l], o1) and torch.equal(krot[l], k1) and torch.equal(lse[l], l1), f"layer {l}"
        ref = O.prefill_attn(W.to_f64(q[l]), W.to_f64(k[l]), W.to_f64(v[l]), cu, pos)
        check_attn(out[l], ref["out"], dtype, f"layer {l} out")
        check_attn(krot[l], ref["k_rot"], dtype, f"layer {l} k_rot")
    assert torch.isnan(out_wide[:, T:].float()).all()     # the rows between the layers were not touched


DECODE_CASES = [
    # dtype, hq, hkv, d, shared lengths, beams, gen_cap, layers
    (BF, 32, 32, 128, [32, 32, 32, 32], 1, 4, 6),       # vector kernel on register caches (MHA)
    (BF, 32, 8, 128, [64, 64], 5, 4, 7),                # matrix-core kernel on register caches with beams
    (BF, 14, 2, 64, [16, 16, 16], 1, 3, 5),             # grouped heads, register caches
    (BF, 8, 2, 128, [900, 129, 2000], 3, 4, 3),         # long caches: key splits + combine, per layer
    (BF, 32, 32, 128, [2059, 700], 1, 3, 2),            # vector kernel with key splits + combine
    (F32, 6, 2, 128, [70, 5], 2, 3, 4),
]


@pytest.mark.parametrize("dtype,hq,hkv,d,slens,beams,gen_cap,n_layers", DECODE_CASES)
def test_decode_layers_equal_single_layer_calls_and_oracle(dtype, hq, hkv, d, slens, beams, gen_cap, n_layers):
    B = _B()
    batch, S, Tt = len(slens), len(slens) * beams, sum(slens)
    g = torch.Generator().manual_seed(Tt + hq + n_layers)
    rnd = lambda *s: torch.randn(*s, generator=g).to(dtype)
    cu = np.concatenate([[0], np.cumsum(slens)]).astype(np.int32)
    s2s = [u // beams for u in range(S)]
    glens = [(u * 2) % gen_cap for u in range(S)]
    q_pos = [slens[s2s[u]] + glens[u] + 11 for u in range(S)]
    L = n_layers
    sk, sv = rnd(L, Tt, hkv, d), rnd(L, Tt, hkv, d)
    q, kn, vn = rnd(L, S, hq, d), rnd(L, S, hkv, d), rnd(L, S, hkv, d)
    gk, gv = rnd(L, S, gen_cap, hkv, d), rnd(L, S, gen_cap, hkv, d)
    desc = B.make_desc(dtype, hq, hkv, d)
    dev = lambda x: x.to(DEV)
    d_gk, d_gv = dev(gk), dev(gv)
    out = torch.full((L, S, hq, d), float("nan"), dtype=dtype, device=DEV)
    args = (dev(q), dev(kn), dev(vn), i32(q_pos), dev(sk), dev(sv), i32(cu), i32(s2s))
    B.earn_decode_attn_layers(desc, *args, d_gk, d_gv, i32(glens), gen_cap, S, batch, max(slens), out)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    ws = torch.empty(max(B.earn_decode_workspace_bytes(desc, S, batch, max(slens), gen_cap), 1), dtype=torch.uint8,
                     device=DEV)
    for l in range(L):
        g1, v1 = dev(gk[l]), dev(gv[l])
        o1 = torch.empty(S, hq, d, dtype=dtype, device=DEV)
        B.earn_decode_attn(desc, args[0][l], args[1][l], args[2][l], args[3], args[4][l], args[5][l], args[6], args[7],
                           g1, v1, i32(glens), gen_cap, S, batch, max(slens), o1, ws)
        torch.cuda.synchronize()
        # same kernels; only the number of key splits may differ between the two launch shapes
        assert torch.equal(d_gk[l], g1) and torch.equal(d_gv[l], v1), f"layer {l} cache append"
        assert (out[l].float() - o1.float()).abs().max() <= (1e-5 if dtype == F32 else 2e-2), f"layer {l}"
        o_gk, o_gv = W.to_f64(gk[l]), W.to_f64(gv[l])
        ref = O.decode_attn(W.to_f64(q[l]), W.to_f64(kn[l]), W.to_f64(vn[l]), q_pos, W.to_f64(sk[l]), W.to_f64(sv[l]), cu,
                            s2s, o_gk, o_gv, glens)
        check_attn(out[l], ref["out"], dtype, f"layer {l} out")
        for u in range(S):
            check_attn(d_gk[l, u, glens[u]], o_gk[u, glens[u]], dtype, f"layer {l} appended key")
            assert torch.equal(d_gv[l, u, glens[u]].cpu(), vn[l, u])


def test_layer_argument_errors():
    B = _B()
    lib = B.lib()
    import ctypes
    fake = ctypes.c_void_p(256)
    desc = B.make_desc(BF, 4, 2, 64)
    call = lambda n_layers=2, qs=1024, ks=512: lib.earn_prefill_attn_layers(
        ctypes.byref(desc), n_layers, fake, qs, fake, fake, ks, fake, None, 1, 8, 8, fake, 1024, fake, 512, None, 0, None, 0,
        None)
    assert call(n_layers=0) == B.EARN_ERR_INVALID_ARG
    assert call(qs=1000) == B.EARN_ERR_INVALID_ARG and b"multiple of 16" in lib.earn_last_error()
    assert call(ks=0) == B.EARN_ERR_INVALID_ARG
    assert call() == B.EARN_ERR_WORKSPACE_TOO_SMALL        # arguments fine, no room for the cos/sin table
    assert lib.earn_prefill_attn_layers(ctypes.byref(desc), 2, fake, 1024, fake, fake, 512, fake, None, 1, 8, 8, fake, 1024,
                                        None, 512, None, 0, None, 0, None) == B.EARN_ERR_INVALID_ARG  # k_rot_out required
    dcall = lambda n_layers=2, gs=4096: lib.earn_decode_attn_layers(
        ctypes.byref(desc), n_layers, fake, 1024, fake, fake, 512, fake, fake, fake, 4096, fake, None, fake, fake, gs, fake,
        4, 2, 2, 100000, 200000, fake, 1024, None, 0, None)
    assert dcall(n_layers=70000) == B.EARN_ERR_INVALID_ARG
    assert dcall(gs=-16) == B.EARN_ERR_INVALID_ARG
    assert dcall() == B.EARN_ERR_WORKSPACE_TOO_SMALL
    assert B.earn_decode_layers_workspace_bytes(desc, 3, 2, 2, 100000, 4) > 0
    assert B.earn_decode_layers_workspace_bytes(desc, 0, 2, 2, 100000, 4) == 0


def test_decode_step_positions():
    B = _B()
    lens = [100, 132, 7]
    cu = i32(np.concatenate([[0], np.cumsum(lens)]))
    s2s = [0, 0, 1, 2, 2, 2]
    q_pos = torch.full((6,), -1, dtype=torch.int32, device=DEV)
    gen_len = torch.full((6,), -1, dtype=torch.int32, device=DEV)
    B.earn_decode_step_positions(cu, i32(s2s), 6, 3, 5, q_pos, gen_len)
    torch.cuda.synchronize()
    assert q_pos.tolist() == [lens[s] + 5 for s in s2s] and gen_len.tolist() == [5] * 6
    q2 = torch.full((3,), -1, dtype=torch.int32, device=DEV)
    B.earn_decode_step_positions(cu, None, 3, 3, 0, q2, None)      # identity map, positions only
    torch.cuda.synchronize()
    assert q2.tolist() == lens
    with pytest.raises(B.EarnError):
        B.earn_decode_step_positions(cu, None, 6, 3, 0, q_pos, gen_len)


def test_whole_path_layer_batched_equals_layer_by_layer():
    """Register-layer prefill and every decode step, once layer by layer and once with the layer-batched calls, on the
    same path object: same outputs (the batched decode may split key ranges differently: tolerance of the bar)."""
    _B()
    from paper_2507_00715_amd.pipeline import EarnPath
    cfg = W.CONFIGS["small_gqa"].replace(batch=4, n_layers=6, split_k=2, decode_steps=3, beams=2)
    w = W.Workload(cfg, history_lengths=[256, 300, 0, 64])
    N, kk, G = cfg.n_layers, cfg.split_k, cfg.decode_steps
    q = [w.prefill_tensor("q", l, device=DEV) for l in range(N)]
    k = [w.prefill_tensor("k", l, device=DEV) for l in range(N)]
    v_full = torch.stack([w.prefill_tensor("v", l, device=DEV) for l in range(kk)])
    v = [v_full[l] if l < kk else w.prefill_tensor("v", l, device=DEV) for l in range(N)]
    dstack = lambda which, g: torch.stack([w.decode_tensor(which, l, g, device=DEV) for l in range(N)])
    dq, dk, dv = ([dstack(t, g) for g in range(G)] for t in "qkv")
    path = EarnPath(n_layers=N, split_k=kk, n_head_reg=cfg.n_head_reg, n_tail_reg=cfg.n_tail_reg,
                    n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim, dtype=cfg.torch_dtype,
                    cu_seqlens=w.cu_seqlens, stream_to_seq=w.stream_to_seq, gen_cap=G, rope_base=cfg.rope_base, device=DEV)
    path.prefill(q, k, v, None)
    torch.cuda.synchronize()
    reg_out, reg_cache = path.reg_prefill_out.clone(), path.reg_k_cache.clone()
    path.reg_prefill_out.fill_(float("nan"))
    path.reg_k_cache.fill_(float("nan"))
    path.bind_prefill_register_layers()()
    torch.cuda.synchronize()
    assert torch.equal(path.reg_prefill_out, reg_out) and torch.equal(path.reg_k_cache, reg_cache)
    path.v_full_stack = v_full
    for g in range(G):
        path.decode_step(g, dq[g], dk[g], dv[g])
        torch.cuda.synchronize()
        want, want_gk = path.decode_out_all.clone(), path.gen_k_all.clone()
        path.decode_out_all.fill_(float("nan"))
        path.gen_k_all[:, :, g] = float("nan")
        path.bind_set_step(g)()
        path.bind_decode_full_layers(dq[g][:kk], dk[g][:kk], dv[g][:kk])()
        path.bind_decode_register_layers(dq[g][kk:], dk[g][kk:], dv[g][kk:])()
        torch.cuda.synchronize()
        assert torch.equal(path.gen_k_all, want_gk)
        assert (path.decode_out_all.float() - want.float()).abs().max() <= 2e-2
