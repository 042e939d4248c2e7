#!/usr/bin/env python3
"""Benchmark of the EARN attention hot path on one MI355X.

A "step" is one pass of the whole path over one synthetic batch of a configuration:
    k full-length prefill layers -> register compaction -> N-k register-only prefill layers -> G decode steps
    (each decode step runs all N layers: full cache for layers < k, register cache for layers >= k).
Inputs are generated on the GPU before the timed region (seeded, synthetic, see paper_2507_00715_amd/workloads.py).

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
# HBM bytes per full-length prefill layer (K rotation + attention kernel), from the rocprofv3 FETCH_SIZE / WRITE_SIZE
# runs summarised in profiles/long_beam_hbm_traffic.txt (counters scaled by a 1 GiB copy: x2.0 and x1.0).
MEASURED_TRAFFIC = {"long_beam": {"fetch_bytes": 3.537e9, "write_bytes": 1.422e9}}
DOMINANT_KERNEL = "prefill_pipe_kernel + rope_k_kernel (one full-length causal layer)"


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
    c = w.cfg
    t0 = time.time()
    seq, pos = w.token_coords(dev)
    mk = lambda which: [w.prefill_tensor(which, l, coords=(seq, pos)) for l in range(c.n_layers)]
    q, k, v = mk("q"), mk("k"), mk("v")
    x = w.prefill_tensor("x", 0, coords=(seq, pos))
    dmk = lambda which: [[w.decode_tensor(which, l, g, device=dev) for l in range(c.n_layers)]
                         for g in range(c.decode_steps)]
    dq, dk, dv = dmk("q"), dmk("k"), dmk("v")
    torch.cuda.synchronize()
    log(f"[bench] {c.name}: inputs generated on GPU in {time.time() - t0:.1f}s "
        f"({torch.cuda.memory_allocated() / 2**30:.1f} GiB allocated)")
    return q, k, v, x, dq, dk, dv


def run_workload(name: str, steps: int, warmup: int, dev) -> dict:
    from paper_2507_00715_amd.pipeline import EarnPath
    cfg = W.CONFIGS[name]
    w = W.Workload(cfg)
    c = cfg
    q, k, v, x, dq, dk, dv = build_inputs(w, dev)
    path = EarnPath(n_layers=c.n_layers, split_k=c.split_k, n_head_reg=c.n_head_reg, n_tail_reg=c.n_tail_reg,
                    n_q_heads=c.n_q_heads, n_kv_heads=c.n_kv_heads, head_dim=c.head_dim, dtype=c.torch_dtype,
                    cu_seqlens=w.cu_seqlens, stream_to_seq=w.stream_to_seq, gen_cap=c.decode_steps,
                    rope_base=c.rope_base, device=dev)
    N, kk, G = c.n_layers, c.split_k, c.decode_steps

    # The launch-bound phases replay the same buffers every step: their calls are marshalled once (the caches of the
    # first k layers are the caller's V tensors, known here; everything else is pre-allocated inside the path).
    for l in range(kk):
        path.v_cache[l] = v[l]
    reg_prefill = [path.bind_prefill_register_layer(l) for l in range(kk, N)]
    dec = [[path.bind_decode_layer(l, dq[g][l], dk[g][l], dv[g][l]) for l in range(N)] for g in range(G)]

    def one_step(tm: PhaseTimer | None):
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
        for call in reg_prefill:
            call()
        pe("prefill_reg")
        for g in range(G):
            path.set_step(g)
            ph("decode_full")
            for l in range(kk):
                dec[g][l]()
            pe("decode_full")
            ph("decode_reg")
            for l in range(kk, N):
                dec[g][l]()
            pe("decode_reg")

    for _ in range(warmup):
        one_step(None)
    torch.cuda.synchronize()
    tm = PhaseTimer()
    t0 = time.perf_counter()
    for _ in range(steps):
        one_step(tm)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms = tm.totals_ms()
    alg = algorithmic_counts(w)

    # Beyond the paper's method, exact: layer k-1 evaluated at the register rows only (its other outputs are dropped by
    # the compaction).  Timed on its own, gather of the query rows included; the timed steps above do not use it.
    rows_only = None
    if 0 < kk < N:
        from paper_2507_00715_amd import binding as B
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
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            rows_layer()
        e1.record()
        torch.cuda.synchronize()
        rows_only = e0.elapsed_time(e1) / reps
        del q_rows, out_rows, ws

    full_ms = ms["prefill_full"] / (steps * kk)              # per launch of the dominant kernel (+ its K rotation)
    reg_ms = ms["prefill_reg"] / (steps * max(N - kk, 1))
    prefill_flops = kk * alg["flops_full"] + (N - kk) * alg["flops_reg"]
    prefill_tflops = prefill_flops * steps / ((ms["prefill_full"] + ms["prefill_reg"]) * 1e-3) / 1e12
    full_tflops = alg["flops_full"] / (full_ms * 1e-3) / 1e12
    dec_bytes_step = [kk * alg["dec_full"][g] + (N - kk) * alg["dec_reg"][g] for g in range(G)]
    dec_ms_total = ms["decode_full"] + ms["decode_reg"]
    dec_us_per_step = dec_ms_total * 1e3 / (steps * G)
    dec_gbps = sum(dec_bytes_step) * steps / (dec_ms_total * 1e-3) / 1e9
    dec_full_gbps = kk * sum(alg["dec_full"]) * steps / (ms["decode_full"] * 1e-3) / 1e9
    dec_reg_gbps = (N - kk) * sum(alg["dec_reg"]) * steps / (ms["decode_reg"] * 1e-3) / 1e9
    comp_us = ms["compact"] * 1e3 / steps
    comp_gbps = alg["compaction"] / (comp_us * 1e-6) / 1e9
    peak = PEAK_BF16_TFLOPS if c.dtype == "bf16" else PEAK_F32_TFLOPS
    res = {
        "workload": w.describe(),
        "ms_per_step": wall * 1e3 / steps,
        "prefill_tflops": prefill_tflops,
        "prefill_full_layer": {"ms_per_launch": full_ms, "tflops": full_tflops, "frac_of_peak": full_tflops / peak,
                               "flops_per_launch": alg["flops_full"],
                               "executed_tile_flops_per_launch": executed_tile_flops(w) if c.dtype == "bf16" else None},
        "prefill_register_layer": {"us_per_launch": reg_ms * 1e3, "flops_per_launch": alg["flops_reg"]},
        "compaction": {"us": comp_us, "bytes": alg["compaction"], "GBps": comp_gbps,
                       "frac_of_hbm_peak": comp_gbps / PEAK_HBM_GBPS},
        "decode": {"us_per_step": dec_us_per_step, "bytes_first_step": dec_bytes_step[0],
                   "bytes_last_step": dec_bytes_step[-1], "GBps": dec_gbps, "frac_of_hbm_peak": dec_gbps / PEAK_HBM_GBPS,
                   "full_cache_layers": {"us_per_layer": ms["decode_full"] * 1e3 / (steps * G * kk),
                                         "GBps": dec_full_gbps, "frac_of_hbm_peak": dec_full_gbps / PEAK_HBM_GBPS},
                   "register_cache_layers": {"us_per_layer": ms["decode_reg"] * 1e3 / (steps * G * max(N - kk, 1)),
                                             "GBps": dec_reg_gbps, "frac_of_hbm_peak": dec_reg_gbps / PEAK_HBM_GBPS}},
        "phase_ms_per_step": {k_: v_ / steps for k_, v_ in ms.items()},
        "last_full_layer_register_rows_only": None if rows_only is None else {
            "ms_per_launch": rows_only, "full_layer_ms_per_launch": ms["prefill_full"] / (steps * kk),
            "ms_per_step_with_it": (wall * 1e3 - ms["prefill_full"] / kk) / steps + rows_only,
            "note": "layer k-1 at the B*r register rows only (gather of the query rows + K rotation + attention); "
                    "exact, beyond the paper's method; not used inside the timed steps"},
        # Context, attention only (not comparable with the paper's end-to-end figures): the same N layers run the
        # vanilla way (every layer full length) would cost N full-layer launches; next to it the closed forms of
        # Section 3.3 (k/N for attention work, (k n + (N-k) r)/(N n) for cache entries).
        "attention_only_vs_vanilla": {
            "prefill_speedup": N * full_ms / (kk * full_ms + (N - kk) * reg_ms),
            "decode_speedup": (N * ms["decode_full"] / max(kk, 1)) / (ms["decode_full"] + ms["decode_reg"]),
            "closed_form_attention_ratio": kk / N,
            "closed_form_cache_ratio": sum(kk * n + (N - kk) * c.r for n in w.seq_lengths) / float(N * sum(w.seq_lengths)),
        },
    }
    del path, q, k, v, x, dq, dk, dv
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
    q0, k0, v0 = (w.prefill_tensor(t, 0, coords=(seq, pos)) for t in "qkv")
    if kind == "prefill_full":
        launch = lambda: path.prefill_full_layer(0, q0, k0, v0)
    elif kind == "decode_full":
        path.prefill_full_layer(0, q0, k0, v0)
        path.set_step(0)
        dq, dk, dv = (w.decode_tensor(t, 0, 0, device=dev) for t in "qkv")
        launch = lambda: path.decode_layer(0, dq, dk, dv)
    elif kind == "compact":
        N, kk = c.n_layers, c.split_k
        mk = lambda which: [w.prefill_tensor(which, l, coords=(seq, pos)) if l >= kk else None for l in range(N)]
        x, q, k, v = w.prefill_tensor("x", 0, coords=(seq, pos)), mk("q"), mk("k"), mk("v")
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default=HEADLINE, choices=W.CONFIG_ORDER)
    ap.add_argument("--others", default="tiny_f32,small_gqa,mid_mha,serving",
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
    floor_us = launch_floor_us(dev)

    cfg = W.CONFIGS[args.workload]
    pf = head["prefill_full_layer"]
    peak = PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else PEAK_F32_TFLOPS
    line = {
        "metric": METRIC,
        "value": head["prefill_tflops"],
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": head["workload"],
        "roofline": {"kernel": DOMINANT_KERNEL, "bound": "mfma",
                     "achieved": pf["tflops"], "peak": peak, "unit": "TFLOP/s", "frac": pf["tflops"] / peak,
                     "traffic": (sum(MEASURED_TRAFFIC[args.workload].values())
                                 if args.workload in MEASURED_TRAFFIC else None),
                     "traffic_detail": MEASURED_TRAFFIC.get(args.workload),
                     "algorithmic_bytes": algorithmic_prefill_bytes(args.workload),
                     "ms_per_launch": pf["ms_per_launch"], "flops_per_launch": pf["flops_per_launch"],
                     "executed_tile_flops_per_launch": pf["executed_tile_flops_per_launch"]},
        "cpu_baseline": cpu,
        "decode": head["decode"],
        "compaction": head["compaction"],
        "prefill_register_layer": head["prefill_register_layer"],
        "phase_ms_per_step": head["phase_ms_per_step"],
        "launch_floor_us": floor_us,
        "last_full_layer_register_rows_only": head["last_full_layer_register_rows_only"],
        "attention_only_vs_vanilla": head["attention_only_vs_vanilla"],
        "other_workloads": {n: {kk: vv for kk, vv in r.items()} for n, r in others.items()},
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
