"""ctypes front end of the fp64 CPU oracle (earn_oracle.c).

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg; never by the product package.  Arrays in and out are numpy fp64 / int32.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "earn_oracle.c")
_LIB = os.path.join(_HERE, "libearn_oracle.so")
_lib = None

c_dp = ctypes.POINTER(ctypes.c_double)
c_ip = ctypes.POINTER(ctypes.c_int32)
c_bp = ctypes.POINTER(ctypes.c_uint8)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP). Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        L.oracle_cache_entries.restype = ctypes.c_int64
        L.oracle_cache_entries.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32,
                                           ctypes.c_int64]
        L.oracle_gamma_cache.restype = ctypes.c_double
        L.oracle_gamma_cache.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_double, ctypes.c_double]
        L.oracle_flops_layer.restype = ctypes.c_double
        L.oracle_flops_layer.argtypes = [ctypes.c_double] * 5
        L.oracle_gamma_attn.restype = ctypes.c_double
        L.oracle_gamma_attn.argtypes = [ctypes.c_int32, ctypes.c_int32] + [ctypes.c_double] * 6
        L.oracle_causal_attn_flops.restype = ctypes.c_double
        L.oracle_causal_attn_flops.argtypes = [c_ip, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32]
        _lib = L
    return _lib


def _d(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(c_dp)


def _i(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(c_ip)


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _i32(a) -> Optional[np.ndarray]:
    return None if a is None else np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"{what}: oracle returned {rc}")


def rope(x, pos, base: float = 10000.0) -> np.ndarray:
    """Rotate x [rows, heads, d] at integer positions pos [rows]."""
    x = _f64(x)
    pos = _i32(pos)
    rows, heads, d = x.shape
    y = np.empty_like(x)
    _check(lib().oracle_rope(_d(x), _i(pos), ctypes.c_int64(rows), heads, d, ctypes.c_double(base), _d(y)), "rope")
    return y


def prefill_attn(q, k, v, cu_seqlens, positions=None, q_to_kv: Optional[Sequence[int]] = None, scale: float = 0.0,
                 rope_base: float = 10000.0, row_sel=None, want_probs: Optional[tuple] = None) -> dict:
    """Causal attention over a packed ragged batch.

    Returns dict(out [T,Hq,d], k_rot [T,Hkv,d], lse [T,Hq], rowsum [T,Hq], probs [n,n] if want_probs=(seq, head)).
    Rows not selected by row_sel hold NaN in out/lse/rowsum.
    """
    q, k, v = _f64(q), _f64(k), _f64(v)
    cu = _i32(cu_seqlens)
    T, hq, d = q.shape
    hkv = k.shape[1]
    assert k.shape == (T, hkv, d) and v.shape == (T, hkv, d) and cu[-1] == T
    batch = len(cu) - 1
    pos = _i32(positions)
    mp = _i32(q_to_kv)
    sel = None if row_sel is None else np.ascontiguousarray(np.asarray(row_sel, dtype=np.uint8))
    out = np.full((T, hq, d), np.nan)
    k_rot = np.empty((T, hkv, d))
    lse = np.full((T, hq), np.nan)
    rowsum = np.full((T, hq), np.nan)
    probs = None
    ps, ph = (-1, -1)
    if want_probs is not None:
        ps, ph = want_probs
        n = int(cu[ps + 1] - cu[ps])
        probs = np.zeros((n, n))
    rc = lib().oracle_prefill_attn(_d(q), _d(k), _d(v), _i(cu), _i(pos), batch, hq, hkv, d, _i(mp),
                                   ctypes.c_double(scale), ctypes.c_double(rope_base),
                                   None if sel is None else sel.ctypes.data_as(c_bp), _d(out), _d(k_rot), _d(lse),
                                   _d(rowsum), _d(probs), ps, ph)
    _check(rc, "prefill_attn")
    res = {"out": out, "k_rot": k_rot, "lse": lse, "rowsum": rowsum}
    if probs is not None:
        res["probs"] = probs
    return res


def compact_registers(src: Optional[np.ndarray], cu_seqlens, n_head_reg: int, n_tail_reg: int) -> dict:
    """Gather the register rows of a packed [T, ...] array (any dtype, bytes are copied).

    Returns dict(dst, idx [B*r], pos [B*r], cu [B+1]); dst is None when src is None.
    """
    cu = _i32(cu_seqlens)
    batch = len(cu) - 1
    r = n_head_reg + n_tail_reg
    idx = np.empty(max(batch * r, 1), dtype=np.int32)
    pos = np.empty(max(batch * r, 1), dtype=np.int32)
    cu_out = np.empty(batch + 1, dtype=np.int32)
    dst = None
    sp = dp = None
    row_bytes = 0
    if src is not None:
        src = np.ascontiguousarray(src)
        assert src.shape[0] == cu[-1]
        row_bytes = src.nbytes // max(src.shape[0], 1)
        dst = np.empty((batch * r,) + src.shape[1:], dtype=src.dtype)
        sp = src.ctypes.data_as(c_bp)
        dp = dst.ctypes.data_as(c_bp)
    rc = lib().oracle_compact_registers(sp, ctypes.c_int64(row_bytes), _i(cu), batch, n_head_reg, n_tail_reg, dp,
                                        _i(idx), _i(pos), _i(cu_out))
    _check(rc, "compact_registers")
    return {"dst": dst, "idx": idx[: batch * r], "pos": pos[: batch * r], "cu": cu_out}


def decode_attn(q, k_new, v_new, q_pos, shared_k, shared_v, shared_cu, stream_to_seq, gen_k: np.ndarray,
                gen_v: np.ndarray, gen_len, q_to_kv=None, scale: float = 0.0, rope_base: float = 10000.0) -> dict:
    """One decode step; gen_k/gen_v [S,gen_cap,Hkv,d] fp64 are updated in place (slot gen_len[u])."""
    q, k_new, v_new = _f64(q), _f64(k_new), _f64(v_new)
    shared_k, shared_v = _f64(shared_k), _f64(shared_v)
    S, hq, d = q.shape
    hkv = k_new.shape[1]
    assert gen_k.dtype == np.float64 and gen_v.dtype == np.float64
    assert gen_k.flags.c_contiguous and gen_v.flags.c_contiguous
    gen_cap = gen_k.shape[1]
    assert gen_k.shape == (S, gen_cap, hkv, d) and gen_v.shape == gen_k.shape
    cu = _i32(shared_cu)
    batch = len(cu) - 1
    assert shared_k.shape[0] == cu[-1]
    out = np.empty((S, hq, d))
    lse = np.empty((S, hq))
    rowsum = np.empty((S, hq))
    rc = lib().oracle_decode_attn(_d(q), _d(k_new), _d(v_new), _i(_i32(q_pos)), _d(shared_k), _d(shared_v), _i(cu),
                                  _i(_i32(stream_to_seq)), _d(gen_k), _d(gen_v), _i(_i32(gen_len)), gen_cap, S, batch,
                                  hq, hkv, d, _i(_i32(q_to_kv)), ctypes.c_double(scale), ctypes.c_double(rope_base),
                                  _d(out), _d(lse), _d(rowsum))
    _check(rc, "decode_attn")
    return {"out": out, "lse": lse, "rowsum": rowsum}


def attn_stats(q, k, cu_seqlens, positions=None, q_to_kv=None, scale: float = 0.0, rope_base: float = 10000.0,
               row_sel=None, epsilon: float = 0.05, t_head: int = 3, tail_back: int = 3) -> np.ndarray:
    """Sparsity, Sink_head, Sink_tail of the causal softmax rows: [T, Hq, 3] (NaN at rows not selected)."""
    q, k = _f64(q), _f64(k)
    cu = _i32(cu_seqlens)
    T, hq, d = q.shape
    hkv = k.shape[1]
    assert k.shape == (T, hkv, d) and cu[-1] == T
    sel = None if row_sel is None else np.ascontiguousarray(np.asarray(row_sel, dtype=np.uint8))
    out = np.full((T, hq, 3), np.nan)
    fn = lib().oracle_attn_stats
    fn.restype = ctypes.c_int
    rc = fn(_d(q), _d(k), _i(cu), _i(_i32(positions)), len(cu) - 1, hq, hkv, d, _i(_i32(q_to_kv)),
            ctypes.c_double(scale), ctypes.c_double(rope_base), None if sel is None else sel.ctypes.data_as(c_bp),
            ctypes.c_double(epsilon), t_head, tail_back, _d(out))
    _check(rc, "attn_stats")
    return out


def beam_topk(beam_scores, token_logprobs, batch: int, beams: int, vocab: int) -> dict:
    """One beam-search selection step: dict(parent [batch*beams] stream index, token, score), best first per sequence."""
    lp = np.ascontiguousarray(np.asarray(token_logprobs, dtype=np.float32)).reshape(batch * beams, vocab)
    bs = None if beam_scores is None else np.ascontiguousarray(np.asarray(beam_scores, dtype=np.float32))
    parent = np.empty(batch * beams, dtype=np.int32)
    token = np.empty(batch * beams, dtype=np.int32)
    score = np.empty(batch * beams, dtype=np.float32)
    c_fp = ctypes.POINTER(ctypes.c_float)
    fn = lib().oracle_beam_topk
    fn.restype = ctypes.c_int
    rc = fn(None if bs is None else bs.ctypes.data_as(c_fp), lp.ctypes.data_as(c_fp), batch, beams, vocab, _i(parent),
            _i(token), score.ctypes.data_as(c_fp))
    _check(rc, "beam_topk")
    return {"parent": parent, "token": token, "score": score}


def beam_reorder_caches(parent, gen_k: np.ndarray, gen_v: np.ndarray) -> None:
    """Beam search by the plain definition: new stream u continues its parent's history, so it takes a COPY of the
    parent's generated cache (in place on gen_k / gen_v [S, gen_cap, Hkv, d])."""
    parent = np.asarray(parent, dtype=np.int64)
    gen_k[...] = gen_k[parent].copy()
    gen_v[...] = gen_v[parent].copy()


def qkv_project(x, w_qkv, n_q_heads: int, n_kv_heads: int, head_dim: int, positions, rope_base: float = 10000.0) -> dict:
    """The Q/K/V projections of a layer (Appendix A.2: X W per head) followed by the rotary embedding of Q and K at the
    rows' original positions.  x [rows, d_model], w_qkv [d_model, (Hq + 2 Hkv) d] with the columns ordered Q heads, K
    heads, V heads.  The matrix product is the library routine in fp64; the rotation is oracle_rope.
    Returns dict(q [rows, Hq, d], k [rows, Hkv, d] (rotated: the cache), v [rows, Hkv, d])."""
    x, w = _f64(x), _f64(w_qkv)
    rows = x.shape[0]
    hq, hkv, d = n_q_heads, n_kv_heads, head_dim
    assert w.shape == (x.shape[1], (hq + 2 * hkv) * d)
    y = x @ w
    q = y[:, : hq * d].reshape(rows, hq, d)
    k = y[:, hq * d: (hq + hkv) * d].reshape(rows, hkv, d)
    v = y[:, (hq + hkv) * d:].reshape(rows, hkv, d)
    pos = _i32(positions)
    return {"q": rope(q, pos, rope_base), "k": rope(k, pos, rope_base), "v": np.ascontiguousarray(v)}


def linear(x, w, activation: int = 0) -> np.ndarray:
    """act(x w): activation 0 = none, 1 = SiLU, y / (1 + exp(-y)) (output projection and the two feed-forward
    projections of Appendix A.2)."""
    y = _f64(x) @ _f64(w)
    return y / (1.0 + np.exp(-y)) if activation == 1 else y


def attn_backward(q, k, v, d_out, cu_seqlens, q_to_kv=None, scale: float = 0.0) -> dict:
    """Gradients of the causal attention with respect to q, k (as the attention saw them: rotated) and v."""
    q, k, v, g = _f64(q), _f64(k), _f64(v), _f64(d_out)
    cu = _i32(cu_seqlens)
    T, hq, d = q.shape
    hkv = k.shape[1]
    dq, dk, dv = np.empty_like(q), np.empty_like(k), np.empty_like(v)
    fn = lib().oracle_attn_backward
    fn.restype = ctypes.c_int
    rc = fn(_d(q), _d(k), _d(v), _d(g), _i(cu), len(cu) - 1, hq, hkv, d, _i(_i32(q_to_kv)), ctypes.c_double(scale),
            _d(dq), _d(dk), _d(dv))
    _check(rc, "attn_backward")
    return {"dq": dq, "dk": dk, "dv": dv}


def cache_entries(n_layers: int, split_k: int, n: int, r: int, gen: int = 0) -> int:
    return int(lib().oracle_cache_entries(n_layers, split_k, n, r, gen))


def gamma_cache(n_layers: int, split_k: int, L: float, r: float) -> float:
    return float(lib().oracle_gamma_cache(n_layers, split_k, L, r))


def flops_layer(L: float, n_h: float, d_a: float, d_h: float, d_f: float) -> float:
    return float(lib().oracle_flops_layer(L, n_h, d_a, d_h, d_f))


def gamma_attn(n_layers: int, split_k: int, L: float, r: float, n_h: float, d_a: float, d_h: float,
               d_f: float) -> float:
    return float(lib().oracle_gamma_attn(n_layers, split_k, L, r, n_h, d_a, d_h, d_f))


def causal_attn_flops(lengths, hq: int, d: int) -> float:
    ln = _i32(lengths)
    return float(lib().oracle_causal_attn_flops(_i(ln), len(ln), hq, d))
