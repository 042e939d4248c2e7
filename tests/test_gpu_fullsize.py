"""Parity at the full sizes of the benchmark configurations, through the same entry points and launch
configurations bench.py times.  The quadratic oracle cannot run a whole layer there, so attention outputs are checked
on SAMPLED rows that the oracle computes one by one (register rows, rows next to tile boundaries, the last row and
random rows of a few (sequence, head) pairs); compaction is checked in full (bit-exact).

Inputs are drawn on the GPU and, for the sampled sequences, again on the CPU from the same counter-based generator
(bit-identical, see test_generator_is_bit_identical_on_cpu_and_gpu), so no oracle input comes from the HIP path.
"""
import numpy as np
import pytest
import torch

from oracle import earn_oracle as O
from paper_2507_00715_amd import workloads as W
from parity import BF16_REL, check_attn, rel_fro, vector_bar

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
BF = torch.bfloat16
BF16_CONFIGS = ["small_gqa", "mid_mha", "long_beam", "serving"]


def _B():
    from paper_2507_00715_amd import binding
    binding.lib()
    return binding


def sample_rows(n, h, t, rng, n_random=24):
    rows = set(range(min(h, n))) | set(range(max(n - t, 0), n))
    for b in (32, 64, 128, 256):
        for k in range(b, n, b * 7 if b < 256 else b):
            rows.update(r for r in (k - 1, k, k + 1) if 0 <= r < n)
    rows.add(n - 1)
    rows.update(int(x) for x in rng.integers(0, n, size=n_random))
    return sorted(rows)


@pytest.mark.parametrize("name", BF16_CONFIGS + ["hstu_prefill"])
def test_full_layer_prefill_sampled_rows(name):
    B = _B()
    cfg = W.CONFIGS[name]
    w = W.Workload(cfg)
    layer = 0
    coords = w.token_coords(DEV)
    q = w.prefill_tensor("q", layer, coords=coords)
    k = w.prefill_tensor("k", layer, coords=coords)
    v = w.prefill_tensor("v", layer, coords=coords)
    out = torch.full_like(q, float("nan"))
    krot = torch.empty_like(k)
    lse = torch.empty(w.total_tokens, cfg.n_q_heads, dtype=torch.float32, device=DEV)
    cu = torch.tensor(w.cu_seqlens, dtype=torch.int32, device=DEV)
    desc = B.make_desc(cfg.torch_dtype, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, 0.0, cfg.rope_base)
    B.earn_prefill_attn(desc, q, k, v, cu, None, cfg.batch, w.total_tokens, w.max_seqlen, out, krot, lse, None)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()

    rng = np.random.default_rng(cfg.config_id)
    lens = np.asarray(w.seq_lengths)
    seqs = sorted({int(np.argmax(lens)), int(np.argmin(lens)), int(rng.integers(0, cfg.batch))})
    gq = cfg.n_q_heads // cfg.n_kv_heads
    worst = 0.0
    for s in seqs:
        n = w.seq_lengths[s]
        b0 = w.cu_seqlens[s]
        heads = sorted({0, cfg.n_q_heads - 1, int(rng.integers(0, cfg.n_q_heads))})
        kvh = sorted({a // gq for a in heads})
        qc = W.to_f64(w.prefill_tensor("q", layer, seqs=[s], heads=heads))
        kc = W.to_f64(w.prefill_tensor("k", layer, seqs=[s], heads=kvh))
        vc = W.to_f64(w.prefill_tensor("v", layer, seqs=[s], heads=kvh))
        rows = sample_rows(n, cfg.n_head_reg, cfg.n_tail_reg, rng)
        sel = np.zeros(n, dtype=np.uint8)
        sel[rows] = 1
        ref = O.prefill_attn(qc, kc, vc, [0, n], q_to_kv=[kvh.index(a // gq) for a in heads], rope_base=cfg.rope_base,
                             row_sel=sel)
        got = out[b0:b0 + n][rows][:, heads].cpu().double().numpy()
        err = check_attn(got, ref["out"][rows], BF, f"{name} seq {s}, {len(rows)} sampled rows",
                         vector_bar(cfg.outlier_scale if cfg.outlier_prob > 0 else 1.0))
        worst = max(worst, err)
        got_lse = lse[b0:b0 + n][rows][:, heads].cpu().double().numpy()
        # log-sum-exp: bf16 operands perturb a score s by about 2^-8 |s|, and the lse follows the largest score
        assert (np.abs(got_lse - ref["lse"][rows]) <= 5e-2 + 1e-2 * np.abs(ref["lse"][rows])).all()
        check_attn(krot[b0:b0 + n][:, kvh], ref["k_rot"], BF, f"{name} seq {s} rotated keys")
    print(f"{name}: worst sampled rel-Frobenius error {worst:.2e}")


def test_prefill_beyond_two_to_the_31_elements():
    """Q and O of more than 2^31 elements (4.4 GB each): the sequence at the far end of the tensors, where 32-bit
    element offsets would have wrapped, against the oracle on sampled rows."""
    B = _B()
    cfg = W.CONFIGS["long_beam"].replace(name="wide", config_id=44, batch=66, len_dist=("fixed", 4096 - 64),
                                         n_q_heads=64, n_kv_heads=8, head_dim=128, beams=1)
    w = W.Workload(cfg)
    assert w.total_tokens * cfg.n_q_heads * cfg.head_dim > 2**31
    coords = w.token_coords(DEV)
    q, k, v = (w.prefill_tensor(t, 0, coords=coords) for t in "qkv")
    out = torch.empty_like(q)
    krot = torch.empty_like(k)
    cu = torch.tensor(w.cu_seqlens, dtype=torch.int32, device=DEV)
    desc = B.make_desc(cfg.torch_dtype, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, 0.0, cfg.rope_base)
    B.earn_prefill_attn(desc, q, k, v, cu, None, cfg.batch, w.total_tokens, w.max_seqlen, out, krot, None, None)
    torch.cuda.synchronize()
    rng = np.random.default_rng(44)
    gq = cfg.n_q_heads // cfg.n_kv_heads
    for s in (cfg.batch - 1, 0):
        n, b0 = w.seq_lengths[s], w.cu_seqlens[s]
        heads = [0, cfg.n_q_heads - 1]
        kvh = sorted({a // gq for a in heads})
        qc = W.to_f64(w.prefill_tensor("q", 0, seqs=[s], heads=heads))
        kc = W.to_f64(w.prefill_tensor("k", 0, seqs=[s], heads=kvh))
        vc = W.to_f64(w.prefill_tensor("v", 0, seqs=[s], heads=kvh))
        rows = sample_rows(n, cfg.n_head_reg, cfg.n_tail_reg, rng, n_random=8)
        sel = np.zeros(n, dtype=np.uint8)
        sel[rows] = 1
        ref = O.prefill_attn(qc, kc, vc, [0, n], q_to_kv=[kvh.index(a // gq) for a in heads], rope_base=cfg.rope_base,
                             row_sel=sel)
        got = out[b0:b0 + n][rows][:, heads].cpu().double().numpy()
        check_attn(got, ref["out"][rows], BF, f"sequence {s}")
        check_attn(krot[b0:b0 + n][:, kvh], ref["k_rot"], BF, f"sequence {s} rotated keys")


@pytest.mark.parametrize("name", BF16_CONFIGS)
def test_full_size_register_rows_of_last_full_layer(name):
    """earn_prefill_register_rows at full size, as bench.py launches it (query rows gathered by earn_compact_registers):
    the register rows of sampled (sequence, head) pairs against the oracle's plain causal attention read at those rows."""
    B = _B()
    cfg = W.CONFIGS[name]
    w = W.Workload(cfg)
    layer, r = cfg.split_k - 1, cfg.r
    coords = w.token_coords(DEV)
    q = w.prefill_tensor("q", layer, coords=coords)
    k = w.prefill_tensor("k", layer, coords=coords)
    v = w.prefill_tensor("v", layer, coords=coords)
    cu = torch.tensor(w.cu_seqlens, dtype=torch.int32, device=DEV)
    q_rows = torch.empty(cfg.batch * r, cfg.n_q_heads, cfg.head_dim, dtype=cfg.torch_dtype, device=DEV)
    idx, pos = (torch.empty(cfg.batch * r, dtype=torch.int32, device=DEV) for _ in range(2))
    cu_c = torch.empty(cfg.batch + 1, dtype=torch.int32, device=DEV)
    B.earn_compact_registers([q], [q_rows], cu, cfg.batch, cfg.n_head_reg, cfg.n_tail_reg, idx, pos, cu_c)
    desc = B.make_desc(cfg.torch_dtype, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, 0.0, cfg.rope_base)
    out = torch.full_like(q_rows, float("nan"))
    krot = torch.empty_like(k)
    ws = torch.empty(max(B.earn_prefill_register_rows_workspace_bytes(desc, cfg.batch, w.max_seqlen, r), 256),
                     dtype=torch.uint8, device=DEV)
    B.earn_prefill_register_rows(desc, q_rows, k, v, cu, pos, cfg.batch, w.total_tokens, w.max_seqlen, r, out, krot, ws)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()

    rng = np.random.default_rng(300 + cfg.config_id)
    lens = np.asarray(w.seq_lengths)
    seqs = sorted({int(np.argmax(lens)), int(np.argmin(lens)), int(rng.integers(0, cfg.batch))})
    gq = cfg.n_q_heads // cfg.n_kv_heads
    for s in seqs:
        n = w.seq_lengths[s]
        heads = sorted({0, cfg.n_q_heads - 1, int(rng.integers(0, cfg.n_q_heads))})
        kvh = sorted({a // gq for a in heads})
        qc = W.to_f64(w.prefill_tensor("q", layer, seqs=[s], heads=heads))
        kc = W.to_f64(w.prefill_tensor("k", layer, seqs=[s], heads=kvh))
        vc = W.to_f64(w.prefill_tensor("v", layer, seqs=[s], heads=kvh))
        rows = list(range(cfg.n_head_reg)) + list(range(n - cfg.n_tail_reg, n))
        sel = np.zeros(n, dtype=np.uint8)
        sel[rows] = 1
        ref = O.prefill_attn(qc, kc, vc, [0, n], q_to_kv=[kvh.index(a // gq) for a in heads], rope_base=cfg.rope_base,
                             row_sel=sel)
        got = out[s * r:(s + 1) * r][:, heads].cpu().double().numpy()
        want = ref["out"][rows]
        check_attn(got, want, BF, f"{name} seq {s}", vector_bar(cfg.outlier_scale if cfg.outlier_prob > 0 else 1.0))
        b0 = w.cu_seqlens[s]
        check_attn(krot[b0:b0 + n][:, kvh], ref["k_rot"], BF, f"{name} seq {s} rotated keys")


@pytest.mark.parametrize("name", BF16_CONFIGS)
def test_full_size_compaction_bit_exact(name):
    """Hidden-state stand-in plus K and V of one later layer, gathered in one launch, against the oracle's indices."""
    B = _B()
    cfg = W.CONFIGS[name]
    w = W.Workload(cfg)
    coords = w.token_coords(DEV)
    x = w.prefill_tensor("x", 0, coords=coords)
    k = w.prefill_tensor("k", cfg.split_k, coords=coords)
    v = w.prefill_tensor("v", cfg.split_k, coords=coords)
    rows = cfg.batch * cfg.r
    dst = [torch.empty((rows,) + tuple(t.shape[1:]), dtype=t.dtype, device=DEV) for t in (x, k, v)]
    idx = torch.empty(rows, dtype=torch.int32, device=DEV)
    pos = torch.empty(rows, dtype=torch.int32, device=DEV)
    cu_c = torch.empty(cfg.batch + 1, dtype=torch.int32, device=DEV)
    cu = torch.tensor(w.cu_seqlens, dtype=torch.int32, device=DEV)
    B.earn_compact_registers([x, k, v], dst, cu, cfg.batch, cfg.n_head_reg, cfg.n_tail_reg, idx, pos, cu_c)
    torch.cuda.synchronize()
    ref = O.compact_registers(None, np.asarray(w.cu_seqlens, dtype=np.int32), cfg.n_head_reg, cfg.n_tail_reg)
    np.testing.assert_array_equal(idx.cpu().numpy(), ref["idx"])
    np.testing.assert_array_equal(pos.cpu().numpy(), ref["pos"])
    np.testing.assert_array_equal(cu_c.cpu().numpy(), ref["cu"])
    # the gathered rows are the source rows the ORACLE's indices name, drawn independently on the CPU
    seq = torch.repeat_interleave(torch.arange(cfg.batch), cfg.r)
    cc = (seq, torch.from_numpy(ref["pos"]).long())
    assert torch.equal(dst[0].cpu(), w.prefill_tensor("x", 0, coords=cc))
    assert torch.equal(dst[1].cpu(), w.prefill_tensor("k", cfg.split_k, coords=cc))
    assert torch.equal(dst[2].cpu(), w.prefill_tensor("v", cfg.split_k, coords=cc))


# "long_beam/20": the long_beam shape at the beam width of the paper's experiments (Appendix, experimental details: beam size 20), 80 query rows per cache
@pytest.mark.parametrize("name,mode", [(n, m) for n in BF16_CONFIGS for m in ("full", "registers")] +
                         [("long_beam/20", "full")])
def test_full_size_decode_sampled_streams(name, mode):
    """One decode step of one layer at full size (full-length cache or register cache), sampled (stream, head) rows."""
    B = _B()
    cfg = W.CONFIGS[name.split("/")[0]]
    if "/" in name:
        cfg = cfg.replace(beams=int(name.split("/")[1]))
    w = W.Workload(cfg)
    layer = 0 if mode == "full" else cfg.split_k
    step = cfg.decode_steps // 2
    G, S = cfg.decode_steps, w.n_streams
    if mode == "full":
        lens, coords_dev = w.seq_lengths, w.token_coords(DEV)
    else:
        lens = [cfg.r] * cfg.batch
        ref_c = O.compact_registers(None, np.asarray(w.cu_seqlens, dtype=np.int32), cfg.n_head_reg, cfg.n_tail_reg)
        seq = torch.repeat_interleave(torch.arange(cfg.batch), cfg.r)
        coords_dev = (seq.to(DEV), torch.from_numpy(ref_c["pos"]).long().to(DEV))
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    # the cache contents stand in for "already rotated keys": drawn, not computed
    sk = w.prefill_tensor("k", layer, coords=coords_dev)
    sv = w.prefill_tensor("v", layer, coords=coords_dev)
    q = w.decode_tensor("q", layer, step, device=DEV)
    kn = w.decode_tensor("k", layer, step, device=DEV)
    vn = w.decode_tensor("v", layer, step, device=DEV)
    # earlier generated rows: draws of the earlier steps (un-rotated draws serve as cache contents)
    gk = torch.zeros(S, G, cfg.n_kv_heads, cfg.head_dim, dtype=cfg.torch_dtype, device=DEV)
    gv = torch.zeros_like(gk)
    for g in range(step):
        gk[:, g] = w.decode_tensor("k", layer, g, device=DEV)
        gv[:, g] = w.decode_tensor("v", layer, g, device=DEV)
    i32 = lambda a: torch.tensor(list(a), dtype=torch.int32, device=DEV)
    q_pos = w.decode_positions(step)
    out = torch.full_like(q, float("nan"))
    desc = B.make_desc(cfg.torch_dtype, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, 0.0, cfg.rope_base)
    ws = torch.empty(max(B.earn_decode_workspace_bytes(desc, S, cfg.batch, max(lens), G), 256), dtype=torch.uint8,
                     device=DEV)
    B.earn_decode_attn(desc, q, kn, vn, i32(q_pos), sk, sv, i32(cu), i32(w.stream_to_seq), gk, gv, i32([step] * S), G, S,
                       cfg.batch, max(lens), out, ws)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()

    rng = np.random.default_rng(100 + cfg.config_id)
    streams = sorted({0, S - 1, *[int(x) for x in rng.integers(0, S, size=4)]})
    gq = cfg.n_q_heads // cfg.n_kv_heads
    for u in streams:
        s = w.stream_to_seq[u]
        n = lens[s]
        heads = sorted({0, cfg.n_q_heads - 1, int(rng.integers(0, cfg.n_q_heads))})
        kvh = sorted({a // gq for a in heads})
        sl = slice(int(cu[s]), int(cu[s]) + n)
        f64 = lambda t: t.cpu().to(torch.float64).numpy()
        # CPU-side inputs of this stream, drawn from the generator (not read back from device buffers)
        if mode == "full":
            cs = w.token_coords("cpu", seqs=[s])
        else:
            cs = (torch.full((cfg.r,), s, dtype=torch.int64), torch.from_numpy(ref_c["pos"][s * cfg.r:(s + 1) * cfg.r]).long())
        skc = W.to_f64(w.prefill_tensor("k", layer, coords=cs, heads=kvh))
        svc = W.to_f64(w.prefill_tensor("v", layer, coords=cs, heads=kvh))
        qc = W.to_f64(w.decode_tensor("q", layer, step, streams=[u])[:, heads])
        knc = W.to_f64(w.decode_tensor("k", layer, step, streams=[u])[:, kvh])
        vnc = W.to_f64(w.decode_tensor("v", layer, step, streams=[u])[:, kvh])
        ogk = np.zeros((1, G, len(kvh), cfg.head_dim))
        ogv = np.zeros_like(ogk)
        for g in range(step):
            ogk[0, g] = W.to_f64(w.decode_tensor("k", layer, g, streams=[u])[:, kvh])[0]
            ogv[0, g] = W.to_f64(w.decode_tensor("v", layer, g, streams=[u])[:, kvh])[0]
        ref = O.decode_attn(qc, knc, vnc, [q_pos[u]], skc, svc, [0, n], None, ogk, ogv, [step],
                            q_to_kv=[kvh.index(a // gq) for a in heads], rope_base=cfg.rope_base)
        check_attn(out[u][heads], ref["out"][0], BF, f"{name}/{mode} stream {u}")
        # cache append
        check_attn(gk[u, step][kvh], ogk[0, step], BF, f"{name}/{mode} stream {u} appended key")
        assert torch.equal(gv[u, step].cpu(), w.decode_tensor("v", layer, step, streams=[u])[0])
        del sl


@pytest.mark.parametrize("mode", ["full", "registers"])
def test_full_size_decode_layer_batched_as_benchmarked(mode):
    """The launch configuration bench.py times on the headline workload: one decode step of ALL full-cache layers (k of
    them) or ALL register-cache layers (N - k) in ONE layer-batched launch at full size; sampled (layer, stream, head)
    rows against the oracle, the appended cache rows included."""
    B = _B()
    cfg = W.CONFIGS["long_beam"]
    w = W.Workload(cfg)
    layers = list(range(cfg.split_k)) if mode == "full" else list(range(cfg.split_k, cfg.n_layers))
    L = len(layers)
    step = cfg.decode_steps // 2
    G, S = cfg.decode_steps, w.n_streams
    if mode == "full":
        lens, coords_dev = w.seq_lengths, w.token_coords(DEV)
    else:
        lens = [cfg.r] * cfg.batch
        ref_c = O.compact_registers(None, np.asarray(w.cu_seqlens, dtype=np.int32), cfg.n_head_reg, cfg.n_tail_reg)
        seq = torch.repeat_interleave(torch.arange(cfg.batch), cfg.r)
        coords_dev = (seq.to(DEV), torch.from_numpy(ref_c["pos"]).long().to(DEV))
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    stack = lambda f: torch.stack([f(l) for l in layers])
    sk = stack(lambda l: w.prefill_tensor("k", l, coords=coords_dev))
    sv = stack(lambda l: w.prefill_tensor("v", l, coords=coords_dev))
    q = stack(lambda l: w.decode_tensor("q", l, step, device=DEV))
    kn = stack(lambda l: w.decode_tensor("k", l, step, device=DEV))
    vn = stack(lambda l: w.decode_tensor("v", l, step, device=DEV))
    gk = torch.zeros(L, S, G, cfg.n_kv_heads, cfg.head_dim, dtype=cfg.torch_dtype, device=DEV)
    gv = torch.zeros_like(gk)
    for i, l in enumerate(layers):
        for g in range(step):
            gk[i, :, g] = w.decode_tensor("k", l, g, device=DEV)
            gv[i, :, g] = w.decode_tensor("v", l, g, device=DEV)
    i32 = lambda a: torch.tensor(list(a), dtype=torch.int32, device=DEV)
    q_pos = w.decode_positions(step)
    out = torch.full_like(q, float("nan"))
    desc = B.make_desc(cfg.torch_dtype, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, 0.0, cfg.rope_base)
    B.earn_decode_attn_layers(desc, q, kn, vn, i32(q_pos), sk, sv, i32(cu), i32(w.stream_to_seq), gk, gv, i32([step] * S), G,
                              S, cfg.batch, max(lens), out)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()

    rng = np.random.default_rng(300 + L)
    gq = cfg.n_q_heads // cfg.n_kv_heads
    for i in sorted({0, L - 1, int(rng.integers(0, L))}):
        l = layers[i]
        for u in sorted({0, S - 1, int(rng.integers(0, S))}):
            s = w.stream_to_seq[u]
            n = lens[s]
            heads = sorted({0, cfg.n_q_heads - 1, int(rng.integers(0, cfg.n_q_heads))})
            kvh = sorted({a // gq for a in heads})
            if mode == "full":
                cs = w.token_coords("cpu", seqs=[s])
            else:
                cs = (torch.full((cfg.r,), s, dtype=torch.int64), torch.from_numpy(ref_c["pos"][s * cfg.r:(s + 1) * cfg.r]).long())
            skc = W.to_f64(w.prefill_tensor("k", l, coords=cs, heads=kvh))
            svc = W.to_f64(w.prefill_tensor("v", l, coords=cs, heads=kvh))
            qc = W.to_f64(w.decode_tensor("q", l, step, streams=[u])[:, heads])
            knc = W.to_f64(w.decode_tensor("k", l, step, streams=[u])[:, kvh])
            vnc = W.to_f64(w.decode_tensor("v", l, step, streams=[u])[:, kvh])
            ogk = np.zeros((1, G, len(kvh), cfg.head_dim))
            ogv = np.zeros_like(ogk)
            for g in range(step):
                ogk[0, g] = W.to_f64(w.decode_tensor("k", l, g, streams=[u])[:, kvh])[0]
                ogv[0, g] = W.to_f64(w.decode_tensor("v", l, g, streams=[u])[:, kvh])[0]
            ref = O.decode_attn(qc, knc, vnc, [q_pos[u]], skc, svc, [0, n], None, ogk, ogv, [step],
                                q_to_kv=[kvh.index(a // gq) for a in heads], rope_base=cfg.rope_base)
            check_attn(out[i, u][heads], ref["out"][0], BF, f"long_beam/{mode} batched layer {l} stream {u}")
            check_attn(gk[i, u, step][kvh], ogk[0, step], BF, f"long_beam/{mode} batched layer {l} stream {u} appended key")
            assert torch.equal(gv[i, u, step].cpu(), w.decode_tensor("v", l, step, streams=[u])[0])


def test_full_size_register_prefill_layer_batched_as_benchmarked():
    """The register-focused prefill layers k..N-1 of the headline workload in ONE layer-batched launch, as bench.py times
    them: compacted sequences of r rows at their original positions; every row of sampled (layer, sequence) pairs against
    the oracle, outputs, rotated keys (the caches) and log-sum-exps."""
    B = _B()
    cfg = W.CONFIGS["long_beam"]
    w = W.Workload(cfg)
    layers = list(range(cfg.split_k, cfg.n_layers))
    L, r, batch = len(layers), cfg.r, cfg.batch
    ref_c = O.compact_registers(None, np.asarray(w.cu_seqlens, dtype=np.int32), cfg.n_head_reg, cfg.n_tail_reg)
    seq = torch.repeat_interleave(torch.arange(batch), r)
    coords_dev = (seq.to(DEV), torch.from_numpy(ref_c["pos"]).long().to(DEV))
    stack = lambda what: torch.stack([w.prefill_tensor(what, l, coords=coords_dev) for l in layers])
    q, k, v = stack("q"), stack("k"), stack("v")
    out, krot = torch.full_like(q, float("nan")), torch.full_like(k, float("nan"))
    lse = torch.full((L, batch * r, cfg.n_q_heads), float("nan"), dtype=torch.float32, device=DEV)
    i32 = lambda a: torch.tensor(np.asarray(a), dtype=torch.int32, device=DEV)
    desc = B.make_desc(cfg.torch_dtype, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, 0.0, cfg.rope_base)
    B.earn_prefill_attn_layers(desc, q, k, v, i32(ref_c["cu"]), i32(ref_c["pos"]), batch, batch * r, r, out, krot, lse)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all() and torch.isfinite(krot.float()).all() and torch.isfinite(lse).all()
    rng = np.random.default_rng(77)
    for i in sorted({0, L - 1, int(rng.integers(0, L))}):
        for s in sorted({0, batch - 1, int(rng.integers(0, batch))}):
            cs = (torch.full((r,), s, dtype=torch.int64), torch.from_numpy(ref_c["pos"][s * r:(s + 1) * r]).long())
            f = lambda what: W.to_f64(w.prefill_tensor(what, layers[i], coords=cs))
            ref = O.prefill_attn(f("q"), f("k"), f("v"), [0, r], positions=ref_c["pos"][s * r:(s + 1) * r],
                                 rope_base=cfg.rope_base)
            sl = slice(s * r, (s + 1) * r)
            check_attn(out[i, sl], ref["out"], BF, f"layer {layers[i]} sequence {s} out")
            check_attn(krot[i, sl], ref["k_rot"], BF, f"layer {layers[i]} sequence {s} rotated keys")
            got_lse = lse[i, sl].cpu().double().numpy()
            assert (np.abs(got_lse - ref["lse"]) <= 5e-2 + 1e-2 * np.abs(ref["lse"])).all()
