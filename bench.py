#!/usr/bin/env python3
"""Benchmark of the EARN attention hot path on one MI355X.

A "step" is one pass of the whole path over one synthetic batch of a configuration:
    k full-length prefill layers -> register compaction -> N-k register-only prefill layers -> G decode steps
    (each decode step runs all N layers: full cache for layers < k, register cache for layers >= k).
Inputs are generated on the GPU before the timed region (seeded, synthetic, see paper_2507_00715_amd/workloads.py).

The timed steps run in the harness throughput mode: the synthetic layers are independent of each other, so the
register-only prefill layers and, per decode step, the k full-cache layers and the N-k register-cache layers each go
out as ONE layer-batched launch (earn_prefill_attn_layers / earn_decode_attn_layers); the full-length prefill layers
stay one launch per layer.  The same steps with one launch per layer (the form a real model needs, where layer l+1
depends on layer l) are timed right after and reported under "per_layer_launch", and once more with those per-layer
launches replayed from HIP graphs ("per_layer_launch_graph").

Prints ONE JSON line.  `value` is the prefill-attention rate in algorithmic causal TFLOP/s
(4*d*Hq*sum_s m_s(m_s+1)/2 per layer, summed over all N prefill launches, divided by the time the prefill
launches took inside the timed steps); decode and compaction figures, a roofline object for the dominant
kernel and the CPU oracle timed on the host cores are carried in the same line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2507_00715_amd import workloads as W  # noqa: E402

METRIC = "prefill attn TFLOP/s + decode attn µs/step & HBM GB/s vs roofline, 1 MI355X"
PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_F32_TFLOPS = 157.3     # fp32 vector
PEAK_HBM_GBPS = 8000.0      # HBM3E
HEADLINE = "long_beam"


def dominant_kernel(cfg, w) -> tuple:
    """Name of the kernel a full-length prefill layer of this workload runs (the library picks by dtype and by the
    lengths: register-sized, medium or long sequences), and the roofline that bounds it."""
    if cfg.dtype != "bf16":
        return "prefill_rows_kernel + rope_k_kernel (one full-length causal layer, vector ALU)", "alu"
    if w.max_seqlen <= 64:
        name = "prefill_mfma_kernel<D,2,1>"
    elif w.max_seqlen <= 3072 or w.total_tokens // cfg.batch <= 2048:
        name = "prefill_mfma_kernel<D,4,2>"
    else:
        name = "prefill_pipe_kernel<D,8>"
    return name + " + rope_k_kernel (one full-length causal layer)", "mfma"


def measured_traffic(name: str):
    """HBM bytes per full-length prefill layer (K rotation + attention kernel) from the rocprofv3 FETCH_SIZE /
    WRITE_SIZE passes: read from the summary profiles/<name>_hbm_traffic.txt, which carries them in one line
    `bench: fetch_bytes=... write_bytes=...` (counters already scaled by what a plain copy of known size reads).
    None when the summary is not there."""
    import re
    path = os.path.join(ROOT, "profiles", f"{name}_hbm_traffic.txt")
    try:
        m = re.search(r"^bench:\s*fetch_bytes=([0-9.e+]+)\s+write_bytes=([0-9.e+]+)", open(path).read(), flags=re.M)
    except OSError:
        return None
    return {"fetch_bytes": float(m.group(1)), "write_bytes": float(m.group(2)), "source": os.path.relpath(path, ROOT)} if m else None


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class PhaseTimer:
    """HIP events on torch's current stream (the stream every libearn launch of this script goes to)."""

    def __init__(self):
        self.pairs = {}

    def start(self, name):
        ev = torch.cuda.Event(enable_timing=True)
        ev.record()
        self.pairs.setdefault(name, []).append([ev, None])

    def stop(self, name):
        ev = torch.cuda.Event(enable_timing=True)
        ev.record()
        self.pairs[name][-1][1] = ev

    def totals_ms(self):
        return {k: sum(a.elapsed_time(b) for a, b in v) for k, v in self.pairs.items()}

    def counts(self):
        return {k: len(v) for k, v in self.pairs.items()}


def algorithmic_counts(w: W.Workload):
    """FLOPs and bytes the method itself requires (not what the kernels happen to move)."""
    c = w.cfg
    e, d, hq, hkv, B, r, S = c.elem_bytes, c.head_dim, c.n_q_heads, c.n_kv_heads, c.batch, c.r, w.n_streams
    flops_full = 4.0 * d * hq * w.causal_pairs(False)
    flops_reg = 4.0 * d * hq * w.causal_pairs(True)
    # decode bytes per layer per step g: K and V rows (shared rows once per sequence) + q,o + k_new,v_new read+write
    def dec_bytes(g, full):
        shared = w.total_tokens if full else B * r
        return 2 * hkv * d * e * (shared + S * (g + 1)) + 2 * hq * d * e * S + 4 * hkv * d * e * S
    dec_full = [dec_bytes(g, True) for g in range(c.decode_steps)]
    dec_reg = [dec_bytes(g, False) for g in range(c.decode_steps)]
    # compaction: x [T, Hq*d] plus q,k,v of the N-k register layers; read + write of B*r rows each, plus index outputs
    row_bytes = [hq * d * e] + [hq * d * e, hkv * d * e, hkv * d * e] * (c.n_layers - c.split_k)
    comp = sum(2 * B * r * rb for rb in row_bytes) + 12 * B * r + 8 * B
    return dict(flops_full=flops_full, flops_reg=flops_reg, dec_full=dec_full, dec_reg=dec_reg, compaction=comp)


def executed_tile_flops(w: W.Workload, tile_keys: int = 64, wave_rows: int = 32) -> float:
    """FLOPs the matrix cores are actually asked for in one full-length layer: every wave of 32 query rows multiplies
    whole 64-key tiles up to and including the tile of its diagonal (masked entries included)."""
    c = w.cfg
    pairs = 0
    for n in w.seq_lengths:
        for q0 in range(0, n, wave_rows):
            pairs += wave_rows * tile_keys * (q0 // tile_keys + 1)
    return 4.0 * c.head_dim * c.n_q_heads * pairs


def algorithmic_prefill_bytes(name: str) -> float:
    """Q, K, V read once, O and the rotated K (the layer's key cache) written once, for one full-length layer."""
    c = W.CONFIGS[name]
    w = W.Workload(c)
    return float(w.total_tokens * c.head_dim * c.elem_bytes * (2 * c.n_q_heads + 3 * c.n_kv_heads))


def build_inputs(w: W.Workload, dev):
    """Per-layer Q, K, V (the values of the first k layers as slices of one [k, T, Hkv, d] tensor, so that their
    decode steps can go out as one launch) and, per decode step, q / k_new / v_new of all layers as [N, S, H, d]."""
    c = w.cfg
    t0 = time.time()
    seq, pos = w.token_coords(dev)
    mk = lambda which: [w.prefill_tensor(which, l, coords=(seq, pos)) for l in range(c.n_layers)]
    q, k = mk("q"), mk("k")
    v_full = torch.empty(c.split_k, w.total_tokens, c.n_kv_heads, c.head_dim, dtype=c.torch_dtype, device=dev)
    v = []
    for l in range(c.n_layers):
        if l < c.split_k:
            v_full[l].copy_(w.prefill_tensor("v", l, coords=(seq, pos)))
            v.append(v_full[l])
        else:
            v.append(w.prefill_tensor("v", l, coords=(seq, pos)))
    x = w.prefill_tensor("x", 0, coords=(seq, pos))
    dmk = lambda which: [torch.stack([w.decode_tensor(which, l, g, device=dev) for l in range(c.n_layers)])
                         for g in range(c.decode_steps)]
    dq, dk, dv = dmk("q"), dmk("k"), dmk("v")
    torch.cuda.synchronize()
    log(f"[bench] {c.name}: inputs generated on GPU in {time.time() - t0:.1f}s "
        f"({torch.cuda.memory_allocated() / 2**30:.1f} GiB allocated)")
    return q, k, v, v_full, x, dq, dk, dv


def run_workload(name: str, steps: int, warmup: int, dev) -> dict:
    from paper_2507_00715_amd.pipeline import EarnPath
    cfg = W.CONFIGS[name]
    w = W.Workload(cfg)
    c = cfg
    q, k, v, v_full, x, dq, dk, dv = build_inputs(w, dev)
    path = EarnPath(n_layers=c.n_layers, split_k=c.split_k, n_head_reg=c.n_head_reg, n_tail_reg=c.n_tail_reg,
                    n_q_heads=c.n_q_heads, n_kv_heads=c.n_kv_heads, head_dim=c.head_dim, dtype=c.torch_dtype,
                    cu_seqlens=w.cu_seqlens, stream_to_seq=w.stream_to_seq, gen_cap=max(c.decode_steps, 1),
                    rope_base=c.rope_base, device=dev)
    N, kk, G = c.n_layers, c.split_k, c.decode_steps       # G = 0: a prefill-only workload

    # The launch-bound phases replay the same buffers every step: their calls are marshalled once (the caches of the
    # first k layers are the caller's V tensors, known here; everything else is pre-allocated inside the path).
    for l in range(kk):
        path.v_cache[l] = v[l]
    path.v_full_stack = v_full
    steps_pos = [path.bind_set_step(g) for g in range(G)]
    # one launch per layer
    reg_prefill = [path.bind_prefill_register_layer(l) for l in range(kk, N)]
    dec = [[path.bind_decode_layer(l, dq[g][l], dk[g][l], dv[g][l]) for l in range(N)] for g in range(G)]
    # one launch per run of independent layers
    reg_prefill_b = path.bind_prefill_register_layers()
    dec_full_b = [path.bind_decode_full_layers(dq[g][:kk], dk[g][:kk], dv[g][:kk]) for g in range(G)]
    dec_reg_b = [path.bind_decode_register_layers(dq[g][kk:], dk[g][kk:], dv[g][kk:]) for g in range(G)]

    # the per-layer launches of the launch-bound phases recorded into HIP graphs (one replay per phase and decode step);
    # the calls read what the prefill and the compaction wrote (caches, compacted bounds and positions): run those first
    from paper_2507_00715_amd.pipeline import capture_graph
    path.prefill(q, k, v, x)
    torch.cuda.synchronize()
    reg_prefill_g = capture_graph(reg_prefill) if N > kk else None
    dec_full_g = [capture_graph([steps_pos[g]] + dec[g][:kk]) for g in range(G)]
    dec_reg_g = [capture_graph(dec[g][kk:]) if N > kk else None for g in range(G)]

    def one_step(tm: PhaseTimer | None, batched, graphs: bool = False):
        ph = (lambda n: tm.start(n)) if tm else (lambda n: None)
        pe = (lambda n: tm.stop(n)) if tm else (lambda n: None)
        ph("prefill_full")
        for l in range(kk):
            path.prefill_full_layer(l, q[l], k[l], v[l])
        pe("prefill_full")
        ph("compact")
        path.compact(x, q, k, v)
        pe("compact")
        ph("prefill_reg")
        if graphs:
            if reg_prefill_g is not None:
                reg_prefill_g.replay()
        elif batched:
            reg_prefill_b()
        else:
            for call in reg_prefill:
                call()
        pe("prefill_reg")
        for g in range(G):
            if not graphs:
                steps_pos[g]()
            ph("decode_full")
            if graphs:
                dec_full_g[g].replay()           # (the step's position update is its first node)
            elif batched:
                dec_full_b[g]()
            else:
                for l in range(kk):
                    dec[g][l]()
            pe("decode_full")
            ph("decode_reg")
            if graphs:
                if dec_reg_g[g] is not None:
                    dec_reg_g[g].replay()
            elif batched:
                dec_reg_b[g]()
            else:
                for l in range(kk, N):
                    dec[g][l]()
            pe("decode_reg")

    def timed(batched: bool, n_steps: int, graphs: bool = False):
        for _ in range(warmup):
            one_step(None, batched, graphs)
        torch.cuda.synchronize()
        tm = PhaseTimer()
        t0 = time.perf_counter()
        for _ in range(n_steps):
            one_step(tm, batched, graphs)
        torch.cuda.synchronize()
        return tm.totals_ms(), time.perf_counter() - t0

    ms, wall = timed(True, steps)
    ms_pl, wall_pl = timed(False, steps)
    ms_gr, wall_gr = timed(False, steps, graphs=True)
    alg = algorithmic_counts(w)

    # The same N layers the vanilla way (Section 3.3's baseline: every layer full length), measured: N full-length
    # prefill launches and N full-cache decode launches, cycling over the tensors of layers 0..k-1.
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for l in range(N):
        path.prefill_full_layer(l % kk, q[l % kk], k[l % kk], v[l % kk])
    e1.record()
    torch.cuda.synchronize()
    vanilla_prefill_ms = e0.elapsed_time(e1)
    vanilla_decode_ms = None
    if G > 0:
        steps_pos[G // 2]()
        e0.record()
        for l in range(N):
            dec[G // 2][l % kk]()
        e1.record()
        torch.cuda.synchronize()
        vanilla_decode_ms = e0.elapsed_time(e1)

    # Attention-score statistics (Sparsity, Sink_head, Sink_tail of the paper's appendix) of the register rows, and of
    # the last row of every sequence alone, over the cache of layer k-1.
    from paper_2507_00715_amd import binding as B
    stats = {}
    if kk > 0:
        l = kk - 1
        q_rows = torch.empty(path.Tc, c.n_q_heads, c.head_dim, dtype=c.torch_dtype, device=dev)
        B.earn_compact_registers([q[l]], [q_rows], path.cu, path.batch, path.h, path.t, path.idx, path.pos, path.cu_c)
        last_pos = torch.tensor([n - 1 for n in w.seq_lengths], dtype=torch.int32, device=dev)
        last_q = q[l][torch.tensor([w.cu_seqlens[s + 1] - 1 for s in range(c.batch)], device=dev)].contiguous()
        for label, rows, qr, pos_t, top in (("register_rows", path.r, q_rows, path.pos, None),
                                           ("last_row", 1, last_q, last_pos, None)):
            out = torch.empty(c.batch * rows, c.n_q_heads, 3, dtype=torch.float32, device=dev)
            call = lambda: B.earn_attn_stats(path.desc, qr, path.k_cache[l], path.cu, pos_t, c.batch, rows, out)
            call()
            torch.cuda.synchronize()
            e0.record()
            for _ in range(5):
                call()
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / 5
            # every key a row can see, once per (sequence, kv head): the longest row of the sequence
            pmax = pos_t.view(c.batch, rows).max(dim=1).values.cpu().tolist()
            nbytes = sum(p_ + 1 for p_ in pmax) * c.n_kv_heads * c.head_dim * c.elem_bytes + qr.numel() * c.elem_bytes + out.numel() * 4
            mean = out.mean(dim=(0, 1)).cpu().tolist()
            stats[label] = {"us": us, "algorithmic_bytes": nbytes, "GBps": nbytes / us / 1e3,
                            "frac_of_hbm_peak": nbytes / us / 1e3 / PEAK_HBM_GBPS,
                            "mean_sparsity_sink_head_sink_tail": mean}
        del q_rows, last_q

    # Beyond the paper's method, exact: layer k-1 evaluated at the register rows only (its other outputs are dropped by
    # the compaction).  Timed on its own, gather of the query rows included; the timed steps above do not use it.
    rows_only = None
    if 0 < kk < N:
        l = kk - 1
        q_rows = torch.empty(path.Tc, c.n_q_heads, c.head_dim, dtype=c.torch_dtype, device=dev)
        out_rows = torch.empty_like(q_rows)
        ws = torch.empty(max(B.earn_prefill_register_rows_workspace_bytes(path.desc, path.batch, path.max_seqlen, path.r),
                             256), dtype=torch.uint8, device=dev)

        def rows_layer():
            B.earn_compact_registers([q[l]], [q_rows], path.cu, path.batch, path.h, path.t, path.idx, path.pos, path.cu_c)
            B.earn_prefill_register_rows(path.desc, q_rows, k[l], v[l], path.cu, path.pos, path.batch, path.T,
                                         path.max_seqlen, path.r, out_rows, path.k_cache[l], ws)
        rows_layer()
        reps = 10
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            rows_layer()
        e1.record()
        torch.cuda.synchronize()
        rows_only = e0.elapsed_time(e1) / reps
        del q_rows, out_rows, ws

    peak = PEAK_BF16_TFLOPS if c.dtype == "bf16" else PEAK_F32_TFLOPS
    dec_bytes_step = [kk * alg["dec_full"][g] + (N - kk) * alg["dec_reg"][g] for g in range(G)]

    def figures(ms, wall):
        full_ms = ms["prefill_full"] / (steps * kk)              # per launch of the dominant kernel (+ its K rotation)
        reg_ms = ms["prefill_reg"] / (steps * max(N - kk, 1))    # per register-only layer
        prefill_flops = kk * alg["flops_full"] + (N - kk) * alg["flops_reg"]
        prefill_tflops = prefill_flops * steps / ((ms["prefill_full"] + ms["prefill_reg"]) * 1e-3) / 1e12
        full_tflops = alg["flops_full"] / (full_ms * 1e-3) / 1e12
        decode = None
        if G > 0:
            dec_ms_total = ms["decode_full"] + ms["decode_reg"]
            dec_gbps = sum(dec_bytes_step) * steps / (dec_ms_total * 1e-3) / 1e9
            dec_full_gbps = kk * sum(alg["dec_full"]) * steps / (ms["decode_full"] * 1e-3) / 1e9
            dec_reg_gbps = (N - kk) * sum(alg["dec_reg"]) * steps / (ms["decode_reg"] * 1e-3) / 1e9
            decode = {"us_per_step": dec_ms_total * 1e3 / (steps * G), "bytes_first_step": dec_bytes_step[0],
                      "bytes_last_step": dec_bytes_step[-1], "GBps": dec_gbps,
                      "frac_of_hbm_peak": dec_gbps / PEAK_HBM_GBPS,
                      "full_cache_layers": {"us_per_layer": ms["decode_full"] * 1e3 / (steps * G * kk),
                                            "GBps": dec_full_gbps, "frac_of_hbm_peak": dec_full_gbps / PEAK_HBM_GBPS},
                      "register_cache_layers": {"us_per_layer": ms["decode_reg"] * 1e3 / (steps * G * max(N - kk, 1)),
                                                "GBps": dec_reg_gbps, "frac_of_hbm_peak": dec_reg_gbps / PEAK_HBM_GBPS}}
        comp_us = ms["compact"] * 1e3 / steps
        comp_gbps = alg["compaction"] / (comp_us * 1e-6) / 1e9
        return {
            "ms_per_step": wall * 1e3 / steps,
            "prefill_tflops": prefill_tflops,
            "prefill_full_layer": {"ms_per_launch": full_ms, "tflops": full_tflops, "frac_of_peak": full_tflops / peak,
                                   "flops_per_launch": alg["flops_full"],
                                   "executed_tile_flops_per_launch": executed_tile_flops(w) if c.dtype == "bf16" else None},
            "prefill_register_layer": {"us_per_layer": reg_ms * 1e3, "flops_per_layer": alg["flops_reg"]},
            "compaction": {"us": comp_us, "bytes": alg["compaction"], "GBps": comp_gbps,
                           "frac_of_hbm_peak": comp_gbps / PEAK_HBM_GBPS},
            "decode": decode,
            "phase_ms_per_step": {k_: v_ / steps for k_, v_ in ms.items()},
        }

    res = {"workload": w.describe(), "launch_mode": "layer-batched register-cache and decode phases"}
    res.update(figures(ms, wall))
    pl = figures(ms_pl, wall_pl)
    res["per_layer_launch"] = {k_: pl[k_] for k_ in ("ms_per_step", "prefill_tflops", "prefill_register_layer", "decode",
                                                     "phase_ms_per_step")}
    gr = figures(ms_gr, wall_gr)
    res["per_layer_launch_graph"] = {k_: gr[k_] for k_ in ("ms_per_step", "prefill_tflops", "prefill_register_layer", "decode",
                                                           "phase_ms_per_step")}
    res["per_layer_launch_graph"]["note"] = ("the per-layer launches of the register prefill and of every decode step "
                                             "replayed from HIP graphs (one launch per layer inside, the form a real "
                                             "model needs)")
    full_ms = res["prefill_full_layer"]["ms_per_launch"]
    res["last_full_layer_register_rows_only"] = None if rows_only is None else {
        "ms_per_launch": rows_only, "full_layer_ms_per_launch": full_ms,
        "ms_per_step_with_it": res["ms_per_step"] - full_ms + rows_only,
        "note": "layer k-1 at the B*r register rows only (gather of the query rows + K rotation + attention); "
                "exact, beyond the paper's method; not used inside the timed steps"}
    # Context, attention only (not comparable with the paper's end-to-end figures): the measured phases against the
    # same N layers run the vanilla way (measured above), next to the closed forms of Section 3.3 (k/N for attention
    # work, (k n + (N-k) r)/(N n) for cache entries).
    earn_prefill_ms = (ms["prefill_full"] + ms["compact"] + ms["prefill_reg"]) / steps
    earn_decode_ms = (ms["decode_full"] + ms["decode_reg"]) / (steps * G) if G > 0 else None
    res["attention_statistics"] = stats
    res["attention_only_vs_vanilla"] = {
        "vanilla_prefill_ms": vanilla_prefill_ms, "earn_prefill_ms": earn_prefill_ms,
        "prefill_speedup": vanilla_prefill_ms / earn_prefill_ms,
        "vanilla_decode_step_ms": vanilla_decode_ms, "earn_decode_step_ms": earn_decode_ms,
        "decode_speedup": vanilla_decode_ms / earn_decode_ms if G > 0 else None,
        "closed_form_attention_ratio": kk / N,
        "closed_form_cache_ratio": sum(kk * n + (N - kk) * c.r for n in w.seq_lengths) / float(N * sum(w.seq_lengths)),
        "note": "vanilla = N full-length prefill launches / N full-cache decode launches (one launch per layer), "
                "measured, cycling over the tensors of layers 0..k-1",
    }
    del path, q, k, v, v_full, x, dq, dk, dv
    torch.cuda.empty_cache()
    return res


def run_single(name: str, kind: str, dev) -> dict:
    """One kernel of the path on its own, launched twice, with as few other dispatches as possible: the form in which
    the hardware-counter passes (rocprofv3 --pmc), which serialise and slow every dispatch, are taken."""
    from paper_2507_00715_amd.pipeline import EarnPath
    c = W.CONFIGS[name]
    w = W.Workload(c)
    seq, pos = w.token_coords(dev)
    path = EarnPath(n_layers=c.n_layers, split_k=c.split_k, n_head_reg=c.n_head_reg, n_tail_reg=c.n_tail_reg,
                    n_q_heads=c.n_q_heads, n_kv_heads=c.n_kv_heads, head_dim=c.head_dim, dtype=c.torch_dtype,
                    cu_seqlens=w.cu_seqlens, stream_to_seq=w.stream_to_seq, gen_cap=c.decode_steps,
                    rope_base=c.rope_base, device=dev)
    q0, k0, v0 = (w.prefill_tensor(t, 0, coords=(seq, pos)) for t in "qkv") if kind != "compact" else (None,) * 3
    if kind == "prefill_full":
        launch = lambda: path.prefill_full_layer(0, q0, k0, v0)
    elif kind == "decode_full":
        path.prefill_full_layer(0, q0, k0, v0)
        path.set_step(0)
        dq, dk, dv = (w.decode_tensor(t, 0, 0, device=dev) for t in "qkv")
        launch = lambda: path.decode_layer(0, dq, dk, dv)
    elif kind == "compact":
        # a byte gather does not care what the bytes are: ONE fill dispatch for all sources (under the counters every
        # dispatch is serialised, and drawing the 85 tensors with the generator took minutes there)
        N, kk = c.n_layers, c.split_k
        T, hq, hkv, d = w.total_tokens, c.n_q_heads, c.n_kv_heads, c.head_dim
        sizes = [T * hq * d] + [T * hq * d, T * hkv * d, T * hkv * d] * (N - kk)
        flat = torch.empty(sum(sizes), dtype=torch.int16, device=dev)
        flat.copy_((torch.arange(flat.numel(), device=dev, dtype=torch.int32) * 40503).to(torch.int16))
        views, off = [], 0
        for sz in sizes:
            views.append(flat[off:off + sz].view(c.torch_dtype))
            off += sz
        x = views[0].view(T, hq * d)
        q = [None] * kk + [views[1 + 3 * i].view(T, hq, d) for i in range(N - kk)]
        k = [None] * kk + [views[2 + 3 * i].view(T, hkv, d) for i in range(N - kk)]
        v = [None] * kk + [views[3 + 3 * i].view(T, hkv, d) for i in range(N - kk)]
        launch = lambda: path.compact(x, q, k, v)
    else:
        raise SystemExit(f"bench.py: unknown --single kind {kind!r}")
    torch.cuda.synchronize()
    launch()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    launch()
    torch.cuda.synchronize()
    return {"workload": name, "single": kind, "launches": 2, "second_launch_ms": (time.perf_counter() - t0) * 1e3}


def launch_floor_us(dev, launches: int = 200) -> float:
    """Cost of one launch through the library with next to no work in it (compaction of one 16-byte row): what every
    per-launch figure of the latency-bound phases contains."""
    from paper_2507_00715_amd import binding as B
    src = torch.zeros(4, 16, dtype=torch.uint8, device=dev)
    dst = torch.zeros(2, 16, dtype=torch.uint8, device=dev)
    cu = torch.tensor([0, 4], dtype=torch.int32, device=dev)
    idx, pos = (torch.zeros(2, dtype=torch.int32, device=dev) for _ in range(2))
    cu_out = torch.zeros(2, dtype=torch.int32, device=dev)
    call = lambda: B.earn_compact_registers([src], [dst], cu, 1, 1, 1, idx, pos, cu_out)
    for _ in range(20):
        call()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(launches):
        call()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / launches


def beam_machinery(name: str, dev, beams: int = 20, vocabs=(256, 32000)) -> dict:
    """Beam search at the paper's beam width on the shape of `name`: the selection step, the ancestor-table update, and
    one decode layer (register cache and full-length cache) reading the generated rows through the table, next to the
    same layer without the table and to the bytes a copy-based reorder of the generated caches would move."""
    from paper_2507_00715_amd import binding as B
    c = W.CONFIGS[name].replace(beams=beams)
    w = W.Workload(c)
    S, G, hq, hkv, d = w.n_streams, c.decode_steps, c.n_q_heads, c.n_kv_heads, c.head_dim
    desc = B.make_desc(c.torch_dtype, hq, hkv, d, 0.0, c.rope_base)
    rnd = lambda *shape: torch.randn(*shape, device=dev, dtype=c.torch_dtype)
    i32 = lambda x: torch.tensor(list(x), dtype=torch.int32, device=dev)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def us(fn, reps=20):
        fn()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / reps

    out = {"beams": beams, "streams": S}
    parent, token = (torch.zeros(S, dtype=torch.int32, device=dev) for _ in range(2))
    scores, new_scores = torch.zeros(S, device=dev), torch.zeros(S, device=dev)
    for V in vocabs:
        lp = torch.randn(S, V, device=dev)
        ws = torch.empty(max(B.earn_beam_topk_workspace_bytes(c.batch, beams, V), 256), dtype=torch.uint8, device=dev)
        t = us(lambda: B.earn_beam_topk(scores, lp, c.batch, beams, V, parent, token, new_scores, ws))
        out[f"topk_vocab_{V}"] = {"us": t, "GBps": S * V * 4 / t / 1e3}
    g = G // 2
    src_a = torch.randint(0, S, (S, G), dtype=torch.int32, device=dev)
    src_a = (src_a % beams + torch.arange(S, device=dev, dtype=torch.int32)[:, None] // beams * beams).contiguous()
    src_b = torch.empty_like(src_a)
    B.earn_beam_topk(scores, torch.randn(S, 256, device=dev), c.batch, beams, 256, parent, token, new_scores)
    out["reorder_table"] = {"us": us(lambda: B.earn_beam_reorder(parent, src_a, src_b, S, G, g)), "bytes": 2 * S * G * 4}
    out["copy_based_reorder_bytes_per_step"] = 2 * 2 * c.n_layers * S * g * hkv * d * c.elem_bytes   # K and V, read + write
    q_pos, gen_len = i32(w.decode_positions(g)), i32([g] * S)
    s2s = i32(w.stream_to_seq)
    for label, lens in (("register_cache_layer", [c.r] * c.batch), ("full_cache_layer", w.seq_lengths)):
        T = sum(lens)
        cu = i32(np.concatenate([[0], np.cumsum(lens)]))
        sk, sv = rnd(T, hkv, d), rnd(T, hkv, d)
        q, kn, vn = rnd(S, hq, d), rnd(S, hkv, d), rnd(S, hkv, d)
        gk, gv = rnd(S, G, hkv, d), rnd(S, G, hkv, d)
        o = torch.empty(S, hq, d, dtype=c.torch_dtype, device=dev)
        ws = torch.empty(max(B.earn_decode_workspace_bytes(desc, S, c.batch, max(lens), G), 256), dtype=torch.uint8, device=dev)
        call = lambda table: B.earn_decode_attn_beams(desc, q, kn, vn, q_pos, sk, sv, cu, s2s, gk, gv, gen_len, table, G, S,
                                                      c.batch, max(lens), o, ws)
        out[label] = {"us_through_table": us(lambda: call(src_b)), "us_without_table": us(lambda: call(None))}
    return out


def decoder_layer(name: str, dev) -> dict:
    """One whole decoder layer in the accounting of the paper's Appendix A.2 (Q/K/V projections with the rotation in
    their epilogue, attention, output projection, two feed-forward projections with SiLU between; no norms or residual
    adds, which the FLOP model leaves out too) at full length and on the compacted register rows, random weights:
    the measured Gamma_attn = (k t_full + (N-k) t_registers) / (N t_full) next to the closed form of Section 3.3."""
    from paper_2507_00715_amd import binding as B
    c = W.CONFIGS[name]
    w = W.Workload(c)
    hq, hkv, d, N, kk = c.n_q_heads, c.n_kv_heads, c.head_dim, c.n_layers, c.split_k
    dm = hq * d
    df = 11008 if dm == 4096 else (int(dm * 2.6875) + 63) // 64 * 64      # the paper's typical values: d_h 4096, d_f 11008
    bf = torch.bfloat16
    g = torch.Generator(device=dev).manual_seed(1)
    rnd = lambda *shape, sc=1.0: (torch.randn(*shape, device=dev, generator=g) * sc).to(bf)
    # weights as [outputs, inputs]
    w_qkv, w_o = rnd((hq + 2 * hkv) * d, dm, sc=dm ** -0.5), rnd(dm, hq * d, sc=dm ** -0.5)
    w_up, w_down = rnd(df, dm, sc=dm ** -0.5), rnd(dm, df, sc=df ** -0.5)
    desc = B.make_desc(bf, hq, hkv, d, 0.0, c.rope_base)
    desc0 = B.make_desc(bf, hq, hkv, d, 0.0, 0.0)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def ms(fn, reps=3):
        fn()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    out = {"d_model": dm, "d_ffn": df}
    r = c.r
    cu_full = torch.tensor(w.cu_seqlens, dtype=torch.int32, device=dev)
    cu_reg = torch.arange(0, c.batch * r + 1, r, dtype=torch.int32, device=dev)
    pos_reg = torch.cat([torch.cat([torch.arange(c.n_head_reg), torch.arange(n - c.n_tail_reg, n)]) for n in w.seq_lengths]).to(torch.int32).to(dev)
    totals = {}
    S = c.batch * max(c.beams, 1)
    pos_dec = torch.tensor([n for n in w.seq_lengths for _ in range(max(c.beams, 1))], dtype=torch.int32, device=dev)
    # few-row products split their inner dimension through this buffer (earn_linear_workspace_bytes)
    lin_ws = torch.empty(max([B.earn_linear_workspace_bytes(rows_, k_, n_) for rows_ in (c.batch * r, S)
                              for k_, n_ in ((dm, (hq + 2 * hkv) * d), (hq * d, dm), (dm, df), (df, dm))] + [256]),
                         dtype=torch.uint8, device=dev)
    for label, rows, cu, pos, maxlen in (("full_length", w.total_tokens, cu_full, None, w.max_seqlen),
                                         ("register_rows", c.batch * r, cu_reg, pos_reg, r),
                                         ("decode_rows", S, None, pos_dec, 0)):
        x = rnd(rows, dm)
        q, k, v = (torch.empty(rows, h_, d, dtype=bf, device=dev) for h_ in (hq, hkv, hkv))
        o, y, hmid = torch.empty(rows, hq, d, dtype=bf, device=dev), torch.empty(rows, dm, dtype=bf, device=dev), torch.empty(rows, df, dtype=bf, device=dev)
        reps = 3 if rows > 4096 else 20
        t = {
            "qkv_rope_project_ms": ms(lambda: B.earn_qkv_rope_project(desc, x, w_qkv, cu, pos, c.batch, q, k, v, lin_ws), reps),
            # (the decode rows' attention is the decode step measured above: not repeated here)
            "attention_ms": ms(lambda: B.earn_prefill_attn(desc0, q, k, v, cu, pos, c.batch, rows, maxlen, o, None, None, None), reps) if maxlen else 0.0,
            "out_projection_ms": ms(lambda: B.earn_linear(o.view(rows, hq * d), w_o, y, 0, lin_ws), reps),
            "ffn_up_silu_ms": ms(lambda: B.earn_linear(x, w_up, hmid, 1, lin_ws), reps),
            "ffn_down_ms": ms(lambda: B.earn_linear(hmid, w_down, y, 0, lin_ws), reps),
        }
        t["layer_ms"] = sum(t.values())
        flops = {"qkv_rope_project": 2.0 * rows * dm * (hq + 2 * hkv) * d, "out_projection": 2.0 * rows * hq * d * dm,
                 "ffn_up_silu": 2.0 * rows * dm * df, "ffn_down": 2.0 * rows * df * dm}
        t["gemm_tflops"] = {k_: flops[k_] / (t[k_ + "_ms"] * 1e-3) / 1e12 for k_ in flops}
        t["gemm_frac_of_bf16_peak"] = {k_: v_ / PEAK_BF16_TFLOPS for k_, v_ in t["gemm_tflops"].items()}
        # context only: the vendor library's GEMM (through torch.matmul) on the feed-forward shape, no activation
        lib_ms = ms(lambda: torch.matmul(x, w_up.t(), out=hmid), reps)
        t["library_matmul_ffn_up_tflops"] = flops["ffn_up_silu"] / (lib_ms * 1e-3) / 1e12
        if rows <= 4096:  # few rows: the weights' bytes are what moves; HBM roofline of the four products together
            wbytes = 2.0 * (dm * (hq + 2 * hkv) * d + hq * d * dm + 2 * dm * df)
            gemm_ms = t["layer_ms"] - t["attention_ms"]
            t["weights_GBps"] = wbytes / (gemm_ms * 1e-3) / 1e9
            t["weights_frac_of_hbm_peak"] = t["weights_GBps"] / PEAK_HBM_GBPS
        out[label] = t
        totals[label] = t["layer_ms"]
        del x, q, k, v, o, y, hmid
    L = sum(w.seq_lengths) / c.batch

    def f_layer(n):  # Appendix A.2: 4 n [n_h d_a (2 d_h + n) + d_h d_f]
        return 4.0 * n * (hq * d * (2 * dm + n) + dm * df)
    out["gamma_attn_measured"] = (kk * totals["full_length"] + (N - kk) * totals["register_rows"]) / (N * totals["full_length"])
    out["gamma_attn_closed_form"] = kk / N + (1 - kk / N) * f_layer(r) / f_layer(L)
    out["k_over_N"] = kk / N
    out["speedup_measured_prefill_layers"] = 1.0 / out["gamma_attn_measured"]
    torch.cuda.empty_cache()
    return out


def attention_backward(name: str, dev) -> dict:
    """earn_attn_backward (vector-ALU form) on the register-focused layers of `name` (compacted sequences of r rows) and
    on one full-length layer of small_gqa: time and the rate of its algorithmic FLOPs, 10 d per causal (query, key) pair
    and head (five products of 2 d: QK^T, dO V^T, P^T dO, dS K, dS^T Q), against the fp32 vector peak."""
    from paper_2507_00715_amd import binding as B
    out = {}
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for label, cname, compacted in (("register_layer", name, True), ("small_gqa_full_layer", "small_gqa", False)):
        c = W.CONFIGS[cname]
        w = W.Workload(c)
        lens = [c.r] * c.batch if compacted else w.seq_lengths
        T = sum(lens)
        rnd = lambda h_: torch.randn(T, h_, c.head_dim, device=dev).to(c.torch_dtype)
        q, k, v, go = rnd(c.n_q_heads), rnd(c.n_kv_heads), rnd(c.n_kv_heads), rnd(c.n_q_heads)
        cu = torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int32, device=dev)
        desc = B.make_desc(c.torch_dtype, c.n_q_heads, c.n_kv_heads, c.head_dim, 0.0, 0.0)
        o = torch.empty_like(q)
        lse = torch.empty(T, c.n_q_heads, dtype=torch.float32, device=dev)
        B.earn_prefill_attn(desc, q, k, v, cu, None, c.batch, T, max(lens), o, None, lse, None)
        dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
        ws = torch.empty(T * c.n_q_heads * 4 + 256, dtype=torch.uint8, device=dev)
        call = lambda: B.earn_attn_backward(desc, q, k, v, o, lse, go, cu, c.batch, T, max(lens), dq, dk, dv, ws)
        call()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(5):
            call()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / 5
        flops = 10.0 * c.head_dim * c.n_q_heads * sum(n * (n + 1) // 2 for n in lens)
        out[label] = {"workload": cname, "us": us, "tflops": flops / us / 1e6, "frac_of_fp32_vector_peak": flops / us / 1e6 / PEAK_F32_TFLOPS,
                      "bound": "alu"}
    return out


def measured_peaks(dev) -> dict:
    """Ceilings measured in this process with the calibration micro-kernels of libearn_calib.so (plain loops, no
    attention code): what the published peaks come to on this machine under this power limit."""
    import ctypes
    from paper_2507_00715_amd import build as earn_build
    if not os.path.exists(earn_build.CALIB_LIB):
        return {"error": "libearn_calib.so not built"}
    L = ctypes.CDLL(earn_build.CALIB_LIB)
    vp = ctypes.c_void_p
    L.earn_calib_sink_floats.restype = ctypes.c_size_t
    L.earn_calib_mfma.argtypes = [vp, ctypes.c_int, ctypes.c_int, vp]
    L.earn_calib_mfma_flops.restype = ctypes.c_double
    L.earn_calib_mfma_flops.argtypes = [ctypes.c_int]
    L.earn_calib_attention_mix.argtypes = [vp, ctypes.c_int, vp]
    L.earn_calib_attention_mix_flops.restype = ctypes.c_double
    L.earn_calib_attention_mix_flops.argtypes = [ctypes.c_int]
    L.earn_calib_attention_mix_rows.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, vp]
    L.earn_calib_attention_mix_rows_flops.restype = ctypes.c_double
    L.earn_calib_attention_mix_rows_flops.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int]
    L.earn_calib_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
    L.earn_calib_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
    sink = torch.zeros(int(L.earn_calib_sink_floats()), dtype=torch.float32, device=dev)
    word = torch.zeros(1, dtype=torch.int32, device=dev)
    nbytes = 1 << 30
    a = torch.full((nbytes // 4,), 0x01010101, dtype=torch.int32, device=dev)
    b = torch.empty_like(a)
    stream = lambda: ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)

    def best_ms(fn, reps=3):
        fn()
        torch.cuda.synchronize()
        best = float("inf")
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            rc = fn()
            e1.record()
            torch.cuda.synchronize()
            assert rc == 0
            best = min(best, e0.elapsed_time(e1))
        return best

    it_mfma, it_mix = 40000, 6000     # 5-20 ms per launch: long enough for the clock to settle under load
    out = {"note": "plain loops timed with HIP events in this process; best of 3 launches each"}
    for label, rnd in (("mfma_bf16_constant_operands_tflops", 0), ("mfma_bf16_random_operands_tflops", 1)):
        ms = best_ms(lambda: L.earn_calib_mfma(vp(sink.data_ptr()), it_mfma, rnd, stream()))
        out[label] = L.earn_calib_mfma_flops(it_mfma) / (ms * 1e-3) / 1e12
    ms = best_ms(lambda: L.earn_calib_attention_mix(vp(sink.data_ptr()), it_mix, stream()))
    out["attention_tile_mix_random_operands_tflops"] = L.earn_calib_attention_mix_flops(it_mix) / (ms * 1e-3) / 1e12
    # the same tile mix in the wave shapes a prefill kernel can take: 32 query rows per wave on one or two waves per
    # SIMD (two = the long-sequence kernel), and 64 rows per wave on one wave per SIMD (half the LDS fragment reads)
    for label, rb, wgs in (("tile_mix_32_rows_per_wave_2_waves_per_simd_tflops", 1, 2),
                           ("tile_mix_32_rows_per_wave_1_wave_per_simd_tflops", 1, 1),
                           ("tile_mix_64_rows_per_wave_1_wave_per_simd_tflops", 2, 1)):
        ms = best_ms(lambda: L.earn_calib_attention_mix_rows(vp(sink.data_ptr()), it_mix, rb, wgs, stream()))
        out[label] = L.earn_calib_attention_mix_rows_flops(it_mix, rb, wgs) / (ms * 1e-3) / 1e12
    ms = best_ms(lambda: L.earn_calib_read(vp(a.data_ptr()), nbytes, vp(word.data_ptr()), stream()))
    out["hbm_read_GBps"] = nbytes / (ms * 1e-3) / 1e9
    ms = best_ms(lambda: L.earn_calib_copy(vp(b.data_ptr()), vp(a.data_ptr()), nbytes, stream()))
    out["hbm_copy_GBps_read_plus_write"] = 2 * nbytes / (ms * 1e-3) / 1e9
    del a, b
    torch.cuda.empty_cache()
    return out


def cpu_baseline_extras(name: str) -> dict:
    """The other oracle functions on bounded samples: one decode step of one full-cache layer of the headline workload
    (the streams of its first sequences), the compaction of its hidden-state stand-in, one full-length prefill layer of
    the small grouped-query configuration in full, and the whole path of the tiny fp32 configuration."""
    from oracle import earn_oracle as O
    from oracle import pipeline as OP
    out = {}
    cfg = W.CONFIGS[name]
    w = W.Workload(cfg)
    # decode: streams of the first two sequences, full-length cache of layer 0, step G/2
    seqs = list(range(min(2, cfg.batch)))
    streams = [u for u in range(w.n_streams) if w.stream_to_seq[u] in seqs]
    g, G = cfg.decode_steps // 2, cfg.decode_steps
    sk = W.to_f64(w.prefill_tensor("k", 0, seqs=seqs))
    sv = W.to_f64(w.prefill_tensor("v", 0, seqs=seqs))
    lens = [w.seq_lengths[s] for s in seqs]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    dq, dk, dv = (W.to_f64(w.decode_tensor(t, 0, g, streams=streams)) for t in "qkv")
    gk = np.zeros((len(streams), G, cfg.n_kv_heads, cfg.head_dim))
    gv = np.zeros_like(gk)
    t0 = time.perf_counter()
    O.decode_attn(dq, dk, dv, [w.seq_lengths[w.stream_to_seq[u]] + g for u in streams], sk, sv, cu,
                  [seqs.index(w.stream_to_seq[u]) for u in streams], gk, gv, [g] * len(streams), rope_base=cfg.rope_base)
    dt = time.perf_counter() - t0
    e = cfg.elem_bytes
    nbytes = 2 * cfg.n_kv_heads * cfg.head_dim * e * (sum(lens) + len(streams) * (g + 1)) + \
        (2 * cfg.n_q_heads + 4 * cfg.n_kv_heads) * cfg.head_dim * e * len(streams)
    out["decode_full_cache_layer"] = {"value": nbytes / dt / 1e9, "unit": "GB/s (algorithmic bytes of the sample)", "seconds": dt,
                                      "sample": f"{name} layer 0, step {g}: the {len(streams)} streams of sequences {seqs}"}
    # compaction of the hidden-state stand-in (all sequences)
    x = w.prefill_tensor("x", 0)
    xb = x.view(torch.uint8).reshape(x.shape[0], -1).numpy()
    t0 = time.perf_counter()
    O.compact_registers(xb, np.asarray(w.cu_seqlens, dtype=np.int32), cfg.n_head_reg, cfg.n_tail_reg)
    dt = time.perf_counter() - t0
    out["compaction"] = {"value": 2 * cfg.batch * cfg.r * xb.shape[1] / dt / 1e9, "unit": "GB/s", "seconds": dt,
                         "sample": f"{name}: hidden-state stand-in [{x.shape[0]}, {x.shape[1]}], {cfg.batch * cfg.r} rows kept"}
    # one full-length layer of small_gqa, in full
    c2 = W.CONFIGS["small_gqa"]
    w2 = W.Workload(c2)
    q2, k2, v2 = (W.to_f64(w2.prefill_tensor(t, 0)) for t in "qkv")
    t0 = time.perf_counter()
    O.prefill_attn(q2, k2, v2, w2.cu_seqlens, rope_base=c2.rope_base)
    dt = time.perf_counter() - t0
    fl = 4.0 * c2.head_dim * c2.n_q_heads * w2.causal_pairs(False)
    out["small_gqa_full_layer"] = {"value": fl / dt / 1e12, "unit": "TFLOP/s", "seconds": dt,
                                   "sample": "small_gqa layer 0, every row of every sequence"}
    # the whole path of tiny_f32
    c1 = W.CONFIGS["tiny_f32"]
    w1 = W.Workload(c1)
    mk = lambda which: [w1.prefill_tensor(which, l) for l in range(c1.n_layers)]
    dmk = lambda which: [[w1.decode_tensor(which, l, gg) for l in range(c1.n_layers)] for gg in range(c1.decode_steps)]
    t0 = time.perf_counter()
    OP.run(n_layers=c1.n_layers, split_k=c1.split_k, n_head_reg=c1.n_head_reg, n_tail_reg=c1.n_tail_reg,
           cu_seqlens=w1.cu_seqlens, q=mk("q"), k=mk("k"), v=mk("v"), x=w1.prefill_tensor("x", 0), dq=dmk("q"), dk=dmk("k"),
           dv=dmk("v"), stream_to_seq=w1.stream_to_seq, rope_base=c1.rope_base)
    out["tiny_f32_whole_path"] = {"value": (time.perf_counter() - t0) * 1e3, "unit": "ms per step (input draws included)",
                                  "sample": "tiny_f32: prefill, compaction and 4 decode steps of all 4 layers"}
    return out


def cpu_baseline(name: str, threads: int = 0, rows_target: int = 4096) -> dict:
    """The fp64 oracle, untuned, on a bounded sample of the headline workload's first prefill layer (threads = 0: all
    the threads OpenMP gives it; otherwise that many, set through the OpenMP runtime the oracle is linked with)."""
    from oracle import earn_oracle as O
    cfg = W.CONFIGS[name]
    w = W.Workload(cfg)
    seq_id = 0
    n = w.seq_lengths[seq_id]
    stride = max(1, n // rows_target)  # 4096 rows: about 10-20 s of oracle time on 16 host cores
    omp = None
    if threads > 0:
        import ctypes
        O.lib()
        omp = ctypes.CDLL("libgomp.so.1")
        before = omp.omp_get_max_threads()
        omp.omp_set_num_threads(threads)
    q = W.to_f64(w.prefill_tensor("q", 0, seqs=[seq_id]))
    k = W.to_f64(w.prefill_tensor("k", 0, seqs=[seq_id]))
    v = W.to_f64(w.prefill_tensor("v", 0, seqs=[seq_id]))
    sel = np.zeros(n, dtype=np.uint8)
    sel[stride - 1::stride] = 1
    rows = np.nonzero(sel)[0]
    pairs = float(np.sum(rows + 1)) * cfg.n_q_heads
    flops = 4.0 * cfg.head_dim * pairs
    t0 = time.perf_counter()
    O.prefill_attn(q, k, v, [0, n], rope_base=cfg.rope_base, row_sel=sel)
    dt = time.perf_counter() - t0
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    if omp is not None:
        omp.omp_set_num_threads(before)
        cores = threads
    cores = min(cores, cfg.n_q_heads)  # the oracle parallelises over (sequence, head)
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle", "seconds": dt,
            "sample": f"{name} layer 0, sequence {seq_id} (n={n}), all {cfg.n_q_heads} query heads, every "
                      f"{stride}th query row ({len(rows)} rows, {pairs:.3g} causal pairs)"}


def cfg_has_decode(name: str) -> bool:
    return W.CONFIGS[name].decode_steps > 0 and W.CONFIGS[name].dtype == "bf16"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default=HEADLINE, choices=W.CONFIG_ORDER)
    ap.add_argument("--others", default="tiny_f32,small_gqa,mid_mha,serving,hstu_prefill",
                    help="comma-separated workloads also measured and reported under 'other_workloads' ('' = none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--single", default="", choices=["", "prefill_full", "decode_full", "compact"],
                    help="launch just this kernel of the workload twice and exit (for hardware-counter passes)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is a single-GPU hot path; --gpus N with N > 1 is not supported "
              "(sequences are independent, so N GPUs would run N independent copies).", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback.", file=sys.stderr)
        sys.exit(3)
    from paper_2507_00715_amd import binding
    binding.lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.single:
        print(json.dumps(run_single(args.workload, args.single, dev)))
        return
    head = run_workload(args.workload, args.steps, args.warmup, dev)
    others = {}
    for name in [s for s in args.others.split(",") if s and s != args.workload]:
        r = run_workload(name, args.steps, args.warmup, dev)
        others[name] = r
    cpu = None if args.no_cpu_baseline else cpu_baseline(args.workload)
    if cpu is not None:  # the same oracle on one thread, on a sixteenth of the rows
        one = cpu_baseline(args.workload, threads=1, rows_target=256)
        cpu["single_thread"] = {k_: one[k_] for k_ in ("value", "unit", "cores", "seconds", "sample")}
        cpu["other_oracle_functions"] = cpu_baseline_extras(args.workload)
    cfg = W.CONFIGS[args.workload]
    floor_us = launch_floor_us(dev)
    peaks = measured_peaks(dev)
    beams20 = beam_machinery(args.workload, dev) if cfg_has_decode(args.workload) else None
    layer = decoder_layer(args.workload, dev) if cfg.dtype == "bf16" else None
    backward = attention_backward(args.workload, dev)

    traffic = measured_traffic(args.workload)
    pf = head["prefill_full_layer"]
    peak = PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else PEAK_F32_TFLOPS
    dominant = dominant_kernel(cfg, W.Workload(cfg))
    line = {
        "metric": METRIC,
        "value": head["prefill_tflops"],
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": dict(head["workload"], launch_mode=head["launch_mode"]),
        "roofline": {"kernel": dominant[0], "bound": dominant[1],
                     "achieved": pf["tflops"], "peak": peak, "unit": "TFLOP/s", "frac": pf["tflops"] / peak,
                     "traffic": None if traffic is None else traffic["fetch_bytes"] + traffic["write_bytes"],
                     "traffic_detail": traffic,
                     "measured_peak": peaks,
                     "algorithmic_bytes": algorithmic_prefill_bytes(args.workload),
                     "ms_per_launch": pf["ms_per_launch"], "flops_per_launch": pf["flops_per_launch"],
                     "executed_tile_flops_per_launch": pf["executed_tile_flops_per_launch"]},
        "cpu_baseline": cpu,
        "decode": head["decode"],
        "compaction": head["compaction"],
        "prefill_register_layer": head["prefill_register_layer"],
        "phase_ms_per_step": head["phase_ms_per_step"],
        "per_layer_launch": head["per_layer_launch"],
        "per_layer_launch_graph": head["per_layer_launch_graph"],
        "attention_statistics": head["attention_statistics"],
        "beam_search_width_20": beams20,
        "decoder_layer_with_projections": layer,
        "attention_backward": backward,
        "launch_floor_us": floor_us,
        "last_full_layer_register_rows_only": head["last_full_layer_register_rows_only"],
        "attention_only_vs_vanilla": head["attention_only_vs_vanilla"],
        "other_workloads": {n: {kk: vv for kk, vv in r.items()} for n, r in others.items()},
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
