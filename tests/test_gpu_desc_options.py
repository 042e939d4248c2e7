"""The fields of earn_attn_desc that the configurations leave at their defaults, on every kernel family, against the
fp64 oracle called with the same options: an explicit softmax scale (Eq. 3's 1/sqrt(d) replaced by 0.37), rotation
switched off (rope_base = 0), and an explicit, permuted grouped-query head map (q_to_kv).

Kernel families reached: bf16 prefill in the 64-row (register layers), 128-row and 256-row (pipelined) forms, the fp32
vector prefill, the vector decode kernel (bf16 and fp32), the matrix-core decode kernel, and the register-rows entry
point in both of its forms.
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


def permuted_map(hq, hkv, seed):
    """A head map that gives every kv head Hq/Hkv query heads, scattered."""
    rng = np.random.default_rng(seed)
    m = np.repeat(np.arange(hkv), hq // hkv)
    rng.shuffle(m)
    return [int(x) for x in m]


# "scale": an explicit scale of the default's order (0.8 / sqrt(d)).  "scale-sharp": 0.37, three to four times the
# default 1/sqrt(d): scores, and with them the absolute score errors that bf16 operands cause (about 2^-9 of a score's
# terms), grow in proportion, the softmax is peaked, and single (row, head) vectors among a thousand reach 2.2e-2 of
# their norm while the tensor stays at 5e-3; those cases keep the tensor-wide 2e-2 and take 4e-2 per vector.
OPTIONS = [
    dict(scale="0.8/sqrt(d)"),
    dict(scale=0.37, vector_bar=4e-2),
    dict(rope_base=0.0),
    dict(q_to_kv="permuted"),
    dict(scale="0.8/sqrt(d)", rope_base=500.0, q_to_kv="permuted"),
]
OPT_IDS = ["scale", "scale-sharp", "no-rope", "head-map", "all-three"]


def resolve(opt, hq, hkv, d):
    o = dict(scale=0.0, rope_base=10000.0, q_to_kv=None, vector_bar=2e-2)
    o.update(opt)
    if o["scale"] == "0.8/sqrt(d)":
        o["scale"] = 0.8 / float(np.sqrt(d))
    if o["q_to_kv"] == "permuted":
        o["q_to_kv"] = permuted_map(hq, hkv, hq * 31 + hkv) if hq > hkv else None
        if hq == hkv and hq > 1:  # one query head per kv head: any permutation is a valid map
            o["q_to_kv"] = [int(x) for x in np.random.default_rng(hq).permutation(hq)]
    return o


def make_desc(B, dtype, hq, hkv, d, o):
    return B.make_desc(dtype, hq, hkv, d, o["scale"], o["rope_base"], o["q_to_kv"])


PREFILL_SHAPES = [
    (BF, 8, 2, 128, [40, 16, 64]),          # one K/V tile per sequence: the register-layer kernel
    (BF, 14, 2, 64, [300, 61, 1000]),       # 128-row workgroups
    (BF, 4, 2, 128, [3300, 1000]),          # long on average (mean > 2048 rows): the pipelined kernel
    (F32, 6, 2, 64, [130, 70]),             # vector kernel
]


@pytest.mark.parametrize("opt", OPTIONS, ids=OPT_IDS)
@pytest.mark.parametrize("dtype,hq,hkv,d,lens", PREFILL_SHAPES)
def test_prefill_options(dtype, hq, hkv, d, lens, opt):
    B = _B()
    o = resolve(opt, hq, hkv, d)
    T, batch = sum(lens), len(lens)
    g = torch.Generator().manual_seed(T + hq)
    rnd = lambda *s: torch.randn(*s, generator=g).to(dtype)
    q, k, v = rnd(T, hq, d), rnd(T, hkv, d), rnd(T, hkv, d)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    desc = make_desc(B, dtype, hq, hkv, d, o)
    out = torch.full((T, hq, d), float("nan"), dtype=dtype, device=DEV)
    krot = torch.empty(T, hkv, d, dtype=dtype, device=DEV)
    lse = torch.empty(T, hq, dtype=torch.float32, device=DEV)
    B.earn_prefill_attn(desc, q.to(DEV), k.to(DEV), v.to(DEV), torch.from_numpy(cu).to(DEV), None, batch, T, max(lens),
                        out, krot, lse, None)
    torch.cuda.synchronize()
    ref = O.prefill_attn(W.to_f64(q), W.to_f64(k), W.to_f64(v), cu, None, o["q_to_kv"], o["scale"], o["rope_base"])
    check_attn(out, ref["out"], dtype, "out", o["vector_bar"])
    check_attn(krot, ref["k_rot"], dtype, "k_rot")
    lse_err = np.abs(lse.cpu().double().numpy() - ref["lse"]).max()
    assert lse_err < (1e-4 if dtype == F32 else 5e-2), f"lse err {lse_err}"
    if o["rope_base"] <= 0:
        assert torch.equal(krot.cpu(), k)


DECODE_SHAPES = [
    # dtype, hq, hkv, d, shared lengths, beams
    (BF, 4, 4, 64, [300, 16, 70], 1),        # vector kernel, one wave
    (BF, 32, 32, 128, [2059, 700], 1),       # vector kernel, long lists, key splits + combine
    (BF, 8, 2, 128, [900, 129], 3),          # matrix-core kernel with beams, key splits + combine
    (BF, 14, 2, 64, [16, 16, 16], 2),        # matrix-core kernel on register-sized caches
    (F32, 6, 2, 128, [70, 5], 2),            # fp32 vector kernel
]


@pytest.mark.parametrize("opt", OPTIONS, ids=OPT_IDS)
@pytest.mark.parametrize("dtype,hq,hkv,d,slens,beams", DECODE_SHAPES)
def test_decode_options(dtype, hq, hkv, d, slens, beams, opt):
    B = _B()
    o = resolve(opt, hq, hkv, d)
    batch, S, gen_cap = len(slens), len(slens) * beams, 4
    g = torch.Generator().manual_seed(sum(slens) + hq)
    rnd = lambda *s: torch.randn(*s, generator=g).to(dtype)
    cu = np.concatenate([[0], np.cumsum(slens)]).astype(np.int32)
    s2s = [u // beams for u in range(S)]
    glens = [u % gen_cap for u in range(S)]
    sk, sv = rnd(int(cu[-1]), hkv, d), rnd(int(cu[-1]), hkv, d)
    q, kn, vn = rnd(S, hq, d), rnd(S, hkv, d), rnd(S, hkv, d)
    gk, gv = rnd(S, gen_cap, hkv, d), rnd(S, gen_cap, hkv, d)
    q_pos = [slens[s2s[u]] + glens[u] for u in range(S)]
    desc = make_desc(B, dtype, hq, hkv, d, o)
    dev = lambda x: x.to(DEV)
    i32 = lambda x: torch.tensor(list(x), dtype=torch.int32, device=DEV)
    d_gk, d_gv = dev(gk), dev(gv)
    out = torch.full((S, hq, d), float("nan"), dtype=dtype, device=DEV)
    ws = torch.empty(max(B.earn_decode_workspace_bytes(desc, S, batch, max(slens), gen_cap), 1), dtype=torch.uint8,
                     device=DEV)
    B.earn_decode_attn(desc, dev(q), dev(kn), dev(vn), i32(q_pos), dev(sk), dev(sv), i32(cu), i32(s2s), d_gk, d_gv,
                       i32(glens), gen_cap, S, batch, max(slens), out, ws)
    torch.cuda.synchronize()
    o_gk, o_gv = W.to_f64(gk), W.to_f64(gv)
    ref = O.decode_attn(W.to_f64(q), W.to_f64(kn), W.to_f64(vn), q_pos, W.to_f64(sk), W.to_f64(sv), cu, s2s, o_gk, o_gv,
                        glens, o["q_to_kv"], o["scale"], o["rope_base"])
    check_attn(out, ref["out"], dtype, "out", o["vector_bar"])
    for u in range(S):
        check_attn(d_gk[u, glens[u]], o_gk[u, glens[u]], dtype, "appended key")
        if o["rope_base"] <= 0:
            assert torch.equal(d_gk[u, glens[u]].cpu(), kn[u])
        assert torch.equal(d_gv[u, glens[u]].cpu(), vn[u])


ROWS_SHAPES = [
    (BF, 8, 2, 128, 4, 4, [300, 64, 1000]),
    (BF, 14, 2, 64, 8, 8, [17, 530]),
    (F32, 6, 2, 64, 3, 2, [100, 40]),
]


@pytest.mark.parametrize("opt", OPTIONS, ids=OPT_IDS)
@pytest.mark.parametrize("dtype,hq,hkv,d,h,t,lens", ROWS_SHAPES)
def test_register_rows_options(dtype, hq, hkv, d, h, t, lens, opt):
    B = _B()
    o = resolve(opt, hq, hkv, d)
    r, batch, T = h + t, len(lens), sum(lens)
    g = torch.Generator().manual_seed(T * 3 + hq)
    rnd = lambda *s: torch.randn(*s, generator=g).to(dtype)
    q, k, v = rnd(T, hq, d), rnd(T, hkv, d), rnd(T, hkv, d)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    ref_c = O.compact_registers(None, cu, h, t)
    q_rows = q[torch.from_numpy(ref_c["idx"]).long()].contiguous()
    desc = make_desc(B, dtype, hq, hkv, d, o)
    out = torch.full((batch * r, hq, d), float("nan"), dtype=dtype, device=DEV)
    k_rot = torch.empty(T, hkv, d, dtype=dtype, device=DEV)
    ws = torch.empty(max(B.earn_prefill_register_rows_workspace_bytes(desc, batch, max(lens), r), 256),
                     dtype=torch.uint8, device=DEV)
    B.earn_prefill_register_rows(desc, q_rows.to(DEV), k.to(DEV), v.to(DEV), torch.from_numpy(cu).to(DEV),
                                 torch.from_numpy(ref_c["pos"]).to(DEV), batch, T, max(lens), r, out, k_rot, ws)
    torch.cuda.synchronize()
    sel = np.zeros(T, dtype=np.uint8)
    sel[ref_c["idx"]] = 1
    ref = O.prefill_attn(W.to_f64(q), W.to_f64(k), W.to_f64(v), cu, None, o["q_to_kv"], o["scale"], o["rope_base"],
                         row_sel=sel)
    check_attn(out, ref["out"][ref_c["idx"]], dtype, "register rows", o["vector_bar"])
    check_attn(k_rot, ref["k_rot"], dtype, "rotated keys")


def test_head_maps_the_kernels_cannot_serve_are_refused():
    B = _B()
    x = torch.zeros(8, 4, 64, dtype=BF, device=DEV)
    kv = torch.zeros(8, 2, 64, dtype=BF, device=DEV)
    cu = torch.tensor([0, 8], dtype=torch.int32, device=DEV)
    call = lambda m: B.earn_prefill_attn(B.make_desc(BF, 4, 2, 64, q_to_kv=m), x, kv, kv, cu, None, 1, 8, 8, x.clone(),
                                         kv.clone(), None, None)
    with pytest.raises(B.EarnError) as e:
        call([0, 0, 0, 1])          # groups of unequal size
    assert e.value.code == B.EARN_ERR_UNSUPPORTED and "unequal" in str(e.value)
    with pytest.raises(B.EarnError) as e:
        call([0, 1, 2, 1])          # kv head out of range
    assert e.value.code == B.EARN_ERR_INVALID_ARG
    call([1, 0, 1, 0])              # a permutation is served
    torch.cuda.synchronize()
