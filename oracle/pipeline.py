"""The whole EARN attention path in oracle terms (TEST INFRASTRUCTURE ONLY).

Follows the inference procedure of Section 3.2: the first k layers attend over every token and cache all of
them; at the input of layer k the register rows are gathered; layers k..N-1 attend over registers only; every
decode step appends its key/value (Eq. 4) and attends over the layer's cache (full for layers < k, registers for
layers >= k) plus the generated tokens.

Inputs are CPU torch tensors in their storage dtype (so the gather can be checked byte for byte); all floating
point work is done by earn_oracle in fp64.
"""
from __future__ import annotations

from typing import Dict, List

import numpy as np
import torch

from . import earn_oracle as O


def _f64(t: torch.Tensor) -> np.ndarray:
    return t.to(torch.float64).contiguous().numpy()


def _bytes(t: torch.Tensor) -> np.ndarray:
    t = t.contiguous()
    return t.view(torch.uint8).reshape(t.shape[0], -1).numpy()


def _gather(t: torch.Tensor, cu, h: int, tl: int) -> torch.Tensor:
    """Byte gather of the register rows of a packed tensor, result in t's dtype."""
    dst = O.compact_registers(_bytes(t), cu, h, tl)["dst"]
    rows = dst.shape[0]
    return torch.from_numpy(dst).view(t.dtype).reshape((rows,) + tuple(t.shape[1:]))


def run(*, n_layers: int, split_k: int, n_head_reg: int, n_tail_reg: int, cu_seqlens: List[int],
        q: List[torch.Tensor], k: List[torch.Tensor], v: List[torch.Tensor], x: torch.Tensor,
        dq: List[List[torch.Tensor]], dk: List[List[torch.Tensor]], dv: List[List[torch.Tensor]],
        stream_to_seq: List[int], rope_base: float = 10000.0, q_to_kv=None, scale: float = 0.0) -> Dict:
    """q/k/v[l]: [T,H,d] for every layer l (full length); dq/dk/dv[g][l]: decode-step inputs [S,H,d]."""
    N, kk, h, tl = n_layers, split_k, n_head_reg, n_tail_reg
    cu = np.asarray(cu_seqlens, dtype=np.int32)
    lens = np.diff(cu)
    B = len(lens)
    S = len(stream_to_seq)
    G = len(dq)
    d = q[0].shape[-1]
    hkv = k[0].shape[1]
    out: Dict = {"prefill_out": [None] * N, "k_cache": [None] * N, "v_cache": [None] * N, "decode_out": []}

    # first k layers: full computation
    for l in range(kk):
        res = O.prefill_attn(_f64(q[l]), _f64(k[l]), _f64(v[l]), cu, None, q_to_kv, scale, rope_base)
        out["prefill_out"][l] = res["out"]
        out["k_cache"][l] = res["k_rot"]
        out["v_cache"][l] = _f64(v[l])

    # register compaction at the input of layer k
    comp = O.compact_registers(_bytes(x), cu, h, tl)
    out["idx"], out["pos"], out["cu_c"] = comp["idx"], comp["pos"], comp["cu"]
    out["x_c"] = torch.from_numpy(comp["dst"]).view(x.dtype).reshape(-1, x.shape[1])
    out["q_c"], out["k_c"], out["v_c"] = {}, {}, {}
    for l in range(kk, N):
        out["q_c"][l] = _gather(q[l], cu, h, tl)
        out["k_c"][l] = _gather(k[l], cu, h, tl)
        out["v_c"][l] = _gather(v[l], cu, h, tl)

    # remaining N-k layers: registers only, original positions
    for l in range(kk, N):
        res = O.prefill_attn(_f64(out["q_c"][l]), _f64(out["k_c"][l]), _f64(out["v_c"][l]), out["cu_c"], out["pos"],
                             q_to_kv, scale, rope_base)
        out["prefill_out"][l] = res["out"]
        out["k_cache"][l] = res["k_rot"]
        out["v_cache"][l] = _f64(out["v_c"][l])

    # decode
    gen_k = [np.zeros((S, max(G, 1), hkv, d)) for _ in range(N)]
    gen_v = [np.zeros((S, max(G, 1), hkv, d)) for _ in range(N)]
    for g in range(G):
        q_pos = np.asarray([lens[stream_to_seq[u]] + g for u in range(S)], dtype=np.int32)
        gen_len = np.full(S, g, dtype=np.int32)
        step = []
        for l in range(N):
            scu = cu if l < kk else out["cu_c"]
            res = O.decode_attn(_f64(dq[g][l]), _f64(dk[g][l]), _f64(dv[g][l]), q_pos, out["k_cache"][l],
                                out["v_cache"][l], scu, stream_to_seq, gen_k[l], gen_v[l], gen_len, q_to_kv, scale,
                                rope_base)
            step.append(res["out"])
        out["decode_out"].append(step)
    out["gen_k"], out["gen_v"] = gen_k, gen_v
    out["cache_entries"] = [O.cache_entries(N, kk, int(lens[s]), h + tl, G) for s in range(B)]
    return out
