"""Thin ctypes binding over libearn.so: same names as the C ABI, argument marshalling only.

Every step of the path runs in the HIP kernels; torch is used for device memory and the current stream.
There is no CPU fallback: if the library is missing or no GPU is present the calls raise.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libearn.so")
_lib = None

EARN_OK = 0
EARN_ERR_INVALID_ARG = -1
EARN_ERR_UNSUPPORTED = -2
EARN_ERR_WORKSPACE_TOO_SMALL = -3
EARN_ERR_HIP = -4
EARN_F32, EARN_BF16 = 0, 1
EARN_MAX_COMPACT_TENSORS = 112

EXPORTS = ["earn_last_error", "earn_version", "earn_prefill_attn", "earn_prefill_workspace_bytes",
           "earn_compact_registers", "earn_decode_attn", "earn_decode_workspace_bytes", "earn_cache_entries",
           "earn_prefill_register_rows", "earn_prefill_register_rows_workspace_bytes", "earn_set_validation",
           "earn_set_tuning", "earn_decode_attn_static", "earn_prefill_attn_layers", "earn_decode_attn_layers",
           "earn_decode_layers_workspace_bytes", "earn_decode_step_positions", "earn_attn_stats", "earn_beam_topk", "earn_beam_topk_workspace_bytes",
           "earn_beam_reorder", "earn_decode_attn_beams", "earn_qkv_rope_project", "earn_linear", "earn_linear_workspace_bytes", "earn_attn_backward",
           "earn_attn_backward_workspace_bytes"]
EARN_STATIC_SCRATCH_BYTES = 8 << 20


class EarnError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libearn error {code}: {msg}")
        self.code = code


class AttnDesc(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("q_to_kv", ctypes.POINTER(ctypes.c_int32)),
                ("softmax_scale", ctypes.c_float), ("rope_base", ctypes.c_float)]


def lib():
    """Load libearn.so (built in-tree by build.py / __graft_entry__.build()). Raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} not built: run `python -m paper_2507_00715_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        L.earn_last_error.restype = ctypes.c_char_p
        L.earn_version.restype = ctypes.c_char_p
        L.earn_prefill_attn.restype = ctypes.c_int
        L.earn_prefill_attn.argtypes = [ctypes.POINTER(AttnDesc), vp, vp, vp, vp, vp, i32, i32, i32, vp, vp, vp, vp, sz, vp]
        L.earn_prefill_workspace_bytes.restype = sz
        L.earn_prefill_workspace_bytes.argtypes = [ctypes.POINTER(AttnDesc), i32, i32, i32, i32]
        L.earn_compact_registers.restype = ctypes.c_int
        L.earn_compact_registers.argtypes = [i32, ctypes.POINTER(vp), ctypes.POINTER(vp),
                                             ctypes.POINTER(ctypes.c_int64), vp, i32, i32, i32, i32, vp, vp, vp, vp]
        L.earn_decode_attn.restype = ctypes.c_int
        L.earn_decode_attn.argtypes = [ctypes.POINTER(AttnDesc), vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32,
                                       i32, i32, i32, vp, vp, sz, vp]
        L.earn_decode_attn_static.restype = ctypes.c_int
        L.earn_decode_attn_static.argtypes = [ctypes.POINTER(AttnDesc), vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32,
                                              i32, i32, i32, i32, vp, vp]
        i64 = ctypes.c_int64
        L.earn_prefill_attn_layers.restype = ctypes.c_int
        L.earn_prefill_attn_layers.argtypes = [ctypes.POINTER(AttnDesc), i32, vp, i64, vp, vp, i64, vp, vp, i32, i32, i32,
                                               vp, i64, vp, i64, vp, i64, vp, sz, vp]
        L.earn_decode_attn_layers.restype = ctypes.c_int
        L.earn_decode_attn_layers.argtypes = [ctypes.POINTER(AttnDesc), i32, vp, i64, vp, vp, i64, vp, vp, vp, i64, vp,
                                              vp, vp, vp, i64, vp, i32, i32, i32, i32, i32, vp, i64, vp, sz, vp]
        L.earn_decode_layers_workspace_bytes.restype = sz
        L.earn_decode_layers_workspace_bytes.argtypes = [ctypes.POINTER(AttnDesc), i32, i32, i32, i32, i32]
        L.earn_decode_step_positions.restype = ctypes.c_int
        L.earn_decode_step_positions.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp]
        L.earn_attn_stats.restype = ctypes.c_int
        L.earn_attn_stats.argtypes = [ctypes.POINTER(AttnDesc), vp, vp, vp, vp, i32, i32, i32, ctypes.c_float, i32, i32, vp,
                                      vp]
        L.earn_beam_topk.restype = ctypes.c_int
        L.earn_beam_topk.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp, vp, sz, vp]
        L.earn_beam_topk_workspace_bytes.restype = sz
        L.earn_beam_topk_workspace_bytes.argtypes = [i32, i32, i32]
        L.earn_beam_reorder.restype = ctypes.c_int
        L.earn_beam_reorder.argtypes = [vp, vp, vp, i32, i32, i32, vp]
        L.earn_decode_attn_beams.restype = ctypes.c_int
        L.earn_decode_attn_beams.argtypes = [ctypes.POINTER(AttnDesc), vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32,
                                             i32, i32, i32, i32, vp, vp, sz, vp]
        L.earn_qkv_rope_project.restype = ctypes.c_int
        L.earn_qkv_rope_project.argtypes = [ctypes.POINTER(AttnDesc), vp, vp, i32, i32, vp, vp, i32, vp, vp, vp, vp, sz, vp]
        L.earn_linear.restype = ctypes.c_int
        L.earn_linear.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, sz, vp]
        L.earn_linear_workspace_bytes.restype = sz
        L.earn_linear_workspace_bytes.argtypes = [i32, i32, i32]
        L.earn_attn_backward.restype = ctypes.c_int
        L.earn_attn_backward.argtypes = [ctypes.POINTER(AttnDesc), vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, vp, vp, vp, vp,
                                         sz, vp]
        L.earn_attn_backward_workspace_bytes.restype = sz
        L.earn_attn_backward_workspace_bytes.argtypes = [ctypes.POINTER(AttnDesc), i32]
        L.earn_prefill_register_rows.restype = ctypes.c_int
        L.earn_prefill_register_rows.argtypes = [ctypes.POINTER(AttnDesc), vp, vp, vp, vp, vp, i32, i32, i32, i32, vp, vp,
                                                 vp, sz, vp]
        L.earn_prefill_register_rows_workspace_bytes.restype = sz
        L.earn_prefill_register_rows_workspace_bytes.argtypes = [ctypes.POINTER(AttnDesc), i32, i32, i32]
        L.earn_decode_workspace_bytes.restype = sz
        L.earn_decode_workspace_bytes.argtypes = [ctypes.POINTER(AttnDesc), i32, i32, i32, i32]
        L.earn_cache_entries.restype = ctypes.c_int64
        L.earn_cache_entries.argtypes = [i32, i32, ctypes.c_int64, i32, ctypes.c_int64]
        L.earn_set_validation.restype = ctypes.c_int
        L.earn_set_validation.argtypes = [ctypes.c_int]
        L.earn_set_tuning.restype = ctypes.c_int
        L.earn_set_tuning.argtypes = [ctypes.c_char_p, i32]
        _lib = L
    return _lib


def last_error() -> str:
    return lib().earn_last_error().decode()


def _check(rc: int):
    if rc != EARN_OK:
        raise EarnError(rc, last_error())


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "libearn takes contiguous device tensors"
    return ctypes.c_void_p(t.data_ptr())


def _rows(t: Optional[torch.Tensor], dim: int = 0) -> int:
    """Rows of a packed tensor as the library is told them (0 for None): the bound it holds sequence bounds inside."""
    return 0 if t is None else int(t.shape[dim])


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def make_desc(dtype: torch.dtype, n_q_heads: int, n_kv_heads: int, head_dim: int, softmax_scale: float = 0.0,
              rope_base: float = 10000.0, q_to_kv: Optional[Sequence[int]] = None) -> AttnDesc:
    code = {torch.float32: EARN_F32, torch.bfloat16: EARN_BF16}.get(dtype, 99)
    desc = AttnDesc(code, n_q_heads, n_kv_heads, head_dim, None, softmax_scale, rope_base)
    if q_to_kv is not None:
        arr = (ctypes.c_int32 * len(q_to_kv))(*q_to_kv)
        desc.q_to_kv = ctypes.cast(arr, ctypes.POINTER(ctypes.c_int32))
        desc._q_to_kv_keepalive = arr  # the struct holds a bare pointer
    return desc


def earn_set_validation(enabled: bool) -> bool:
    """Debug validation of device-side preconditions (synchronises the stream on every call). Returns the old setting."""
    return bool(lib().earn_set_validation(int(bool(enabled))))


def earn_set_tuning(key: str, value: int) -> None:
    _check(lib().earn_set_tuning(key.encode(), int(value)))


def earn_prefill_workspace_bytes(desc: AttnDesc, batch: int, total_tokens: int, max_seqlen: int,
                                 have_k_rot_out: bool) -> int:
    return int(lib().earn_prefill_workspace_bytes(ctypes.byref(desc), batch, total_tokens, max_seqlen,
                                                  int(have_k_rot_out)))


def earn_prefill_attn(desc: AttnDesc, q, k, v, cu_seqlens, positions, batch: int, total_tokens: int, max_seqlen: int,
                      out, k_rot_out=None, lse_out=None, workspace=None) -> None:
    if workspace is None:  # convenience for one-off calls; loops pass a buffer sized with earn_prefill_workspace_bytes
        need = earn_prefill_workspace_bytes(desc, batch, total_tokens, max_seqlen, k_rot_out is not None)
        if need:
            workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().earn_prefill_attn(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(cu_seqlens), _ptr(positions),
                                   batch, total_tokens, max_seqlen, _ptr(out), _ptr(k_rot_out), _ptr(lse_out),
                                   _ptr(workspace), ws_bytes, _stream()))


def earn_compact_registers(src: Sequence[torch.Tensor], dst: Sequence[torch.Tensor], cu_seqlens, batch: int,
                           n_head_reg: int, n_tail_reg: int, idx_out=None, pos_out=None, cu_out=None,
                           row_bytes: Optional[Sequence[int]] = None) -> None:
    n = len(src)
    assert len(dst) == n
    vp = ctypes.c_void_p
    src_arr = (vp * max(n, 1))(*[t.data_ptr() for t in src])
    dst_arr = (vp * max(n, 1))(*[t.data_ptr() for t in dst])
    if row_bytes is None:
        row_bytes = [t[0].numel() * t.element_size() if t.shape[0] > 0 else 16 for t in src]
    rb_arr = (ctypes.c_int64 * max(n, 1))(*row_bytes)
    for t in list(src) + list(dst):
        assert t.is_cuda and t.is_contiguous()
    total = min(t.shape[0] for t in src) if n else 0x7fffffff   # no tensors: indices only, nothing is read
    _check(lib().earn_compact_registers(n, src_arr, dst_arr, rb_arr, _ptr(cu_seqlens), batch, total, n_head_reg, n_tail_reg,
                                        _ptr(idx_out), _ptr(pos_out), _ptr(cu_out), _stream()))


def earn_prefill_register_rows_workspace_bytes(desc: AttnDesc, batch: int, max_seqlen: int, rows_per_seq: int) -> int:
    return int(lib().earn_prefill_register_rows_workspace_bytes(ctypes.byref(desc), batch, max_seqlen, rows_per_seq))


def earn_prefill_register_rows(desc: AttnDesc, q_rows, k, v, cu_seqlens, row_pos, batch: int, total_tokens: int,
                               max_seqlen: int, rows_per_seq: int, out_rows, k_rot_out, workspace=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().earn_prefill_register_rows(ctypes.byref(desc), _ptr(q_rows), _ptr(k), _ptr(v), _ptr(cu_seqlens),
                                            _ptr(row_pos), batch, total_tokens, max_seqlen, rows_per_seq,
                                            _ptr(out_rows), _ptr(k_rot_out), _ptr(workspace), ws_bytes, _stream()))


def earn_decode_workspace_bytes(desc: AttnDesc, n_streams: int, batch: int, max_shared_len: int, gen_cap: int) -> int:
    return int(lib().earn_decode_workspace_bytes(ctypes.byref(desc), n_streams, batch, max_shared_len, gen_cap))


def earn_decode_attn(desc: AttnDesc, q, k_new, v_new, q_pos, shared_k, shared_v, shared_cu, stream_to_seq, gen_k,
                     gen_v, gen_len, gen_cap: int, n_streams: int, batch: int, max_shared_len: int, out,
                     workspace=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().earn_decode_attn(ctypes.byref(desc), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(q_pos), _ptr(shared_k),
                                  _ptr(shared_v), _ptr(shared_cu), _ptr(stream_to_seq), _ptr(gen_k), _ptr(gen_v),
                                  _ptr(gen_len), gen_cap, n_streams, batch, max_shared_len, _rows(shared_k), _ptr(out),
                                  _ptr(workspace), ws_bytes, _stream()))


def earn_decode_attn_static(desc: AttnDesc, q, k_new, v_new, q_pos, shared_k, shared_v, shared_cu, stream_to_seq,
                            gen_k, gen_v, gen_len, gen_cap: int, n_streams: int, batch: int, max_shared_len: int,
                            out) -> None:
    """earn_decode_attn without a workspace: partial results go to the library's own per-GPU buffer."""
    _check(lib().earn_decode_attn_static(ctypes.byref(desc), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(q_pos),
                                         _ptr(shared_k), _ptr(shared_v), _ptr(shared_cu), _ptr(stream_to_seq),
                                         _ptr(gen_k), _ptr(gen_v), _ptr(gen_len), gen_cap, n_streams, batch,
                                         max_shared_len, _rows(shared_k), _ptr(out), _stream()))


class BoundCall:
    """An entry-point call with its arguments marshalled ONCE: calling the object enqueues the launch on the stream
    that is current at that moment.  For loops that repeat a call on the same buffers (a decode step per layer on
    pre-allocated caches), where converting a dozen tensors to pointers costs more host time than the launch itself.
    The object keeps the tensors alive."""
    __slots__ = ("_fn", "_args", "_keep")

    def __init__(self, fn, args, keep):
        self._fn, self._args, self._keep = fn, args, keep

    def __call__(self) -> None:
        rc = self._fn(*self._args, torch.cuda.current_stream().cuda_stream)
        if rc != EARN_OK:
            raise EarnError(rc, last_error())


def bind_decode_attn(desc: AttnDesc, q, k_new, v_new, q_pos, shared_k, shared_v, shared_cu, stream_to_seq, gen_k, gen_v,
                     gen_len, gen_cap: int, n_streams: int, batch: int, max_shared_len: int, out,
                     workspace=None) -> BoundCall:
    """earn_decode_attn with the same arguments, marshalled once (see BoundCall)."""
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    tensors = (q, k_new, v_new, q_pos, shared_k, shared_v, shared_cu, stream_to_seq, gen_k, gen_v, gen_len)
    args = (ctypes.byref(desc), *[_ptr(t) for t in tensors], gen_cap, n_streams, batch, max_shared_len, _rows(shared_k),
            _ptr(out), _ptr(workspace), ws_bytes)
    return BoundCall(lib().earn_decode_attn, args, (desc, tensors, out, workspace))


def bind_prefill_attn(desc: AttnDesc, q, k, v, cu_seqlens, positions, batch: int, total_tokens: int, max_seqlen: int,
                      out, k_rot_out, lse_out, workspace) -> BoundCall:
    """earn_prefill_attn with the same arguments (workspace required if the call needs one), marshalled once."""
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    tensors = (q, k, v, cu_seqlens, positions)
    args = (ctypes.byref(desc), *[_ptr(t) for t in tensors], batch, total_tokens, max_seqlen, _ptr(out),
            _ptr(k_rot_out), _ptr(lse_out), _ptr(workspace), ws_bytes)
    return BoundCall(lib().earn_prefill_attn, args, (desc, tensors, out, k_rot_out, lse_out, workspace))


def earn_decode_step_positions(cu_seqlens, stream_to_seq, n_streams: int, batch: int, step: int, q_pos,
                               gen_len) -> None:
    _check(lib().earn_decode_step_positions(_ptr(cu_seqlens), _ptr(stream_to_seq), n_streams, batch, step, _ptr(q_pos),
                                            _ptr(gen_len), _stream()))


def bind_decode_step_positions(cu_seqlens, stream_to_seq, n_streams: int, batch: int, step: int, q_pos,
                               gen_len) -> "BoundCall":
    args = (_ptr(cu_seqlens), _ptr(stream_to_seq), n_streams, batch, step, _ptr(q_pos), _ptr(gen_len))
    return BoundCall(lib().earn_decode_step_positions, args, (cu_seqlens, stream_to_seq, q_pos, gen_len))


def earn_attn_stats(desc: AttnDesc, q_rows, k_rot, cu_seqlens, row_pos, batch: int, rows_per_seq: int, stats_out,
                    epsilon: float = 0.05, t_head: int = 3, tail_back: int = 3) -> None:
    _check(lib().earn_attn_stats(ctypes.byref(desc), _ptr(q_rows), _ptr(k_rot), _ptr(cu_seqlens), _ptr(row_pos), batch,
                                 _rows(k_rot), rows_per_seq, epsilon, t_head, tail_back, _ptr(stats_out), _stream()))


def earn_beam_topk_workspace_bytes(batch: int, beams: int, vocab: int) -> int:
    return int(lib().earn_beam_topk_workspace_bytes(batch, beams, vocab))


def earn_beam_topk(beam_scores, token_logprobs, batch: int, beams: int, vocab: int, parent_out, token_out, score_out,
                   workspace=None) -> None:
    if workspace is None:
        need = earn_beam_topk_workspace_bytes(batch, beams, vocab)
        workspace = torch.empty(need, dtype=torch.uint8, device=token_logprobs.device) if need else None
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().earn_beam_topk(_ptr(beam_scores), _ptr(token_logprobs), batch, beams, vocab, _ptr(parent_out),
                                _ptr(token_out), _ptr(score_out), _ptr(workspace), ws_bytes, _stream()))


def earn_beam_reorder(parent, gen_src_in, gen_src_out, n_streams: int, gen_cap: int, step: int) -> None:
    _check(lib().earn_beam_reorder(_ptr(parent), _ptr(gen_src_in), _ptr(gen_src_out), n_streams, gen_cap, step, _stream()))


def earn_decode_attn_beams(desc: AttnDesc, q, k_new, v_new, q_pos, shared_k, shared_v, shared_cu, stream_to_seq, gen_k,
                           gen_v, gen_len, gen_src, gen_cap: int, n_streams: int, batch: int, max_shared_len: int, out,
                           workspace=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().earn_decode_attn_beams(ctypes.byref(desc), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(q_pos),
                                        _ptr(shared_k), _ptr(shared_v), _ptr(shared_cu), _ptr(stream_to_seq), _ptr(gen_k),
                                        _ptr(gen_v), _ptr(gen_len), _ptr(gen_src), gen_cap, n_streams, batch,
                                        max_shared_len, _rows(shared_k), _ptr(out), _ptr(workspace), ws_bytes, _stream()))


def earn_linear_workspace_bytes(rows: int, k: int, n: int) -> int:
    return int(lib().earn_linear_workspace_bytes(rows, k, n))


def _linear_workspace(rows: int, k: int, n: int, workspace, device):
    """workspace = "auto": allocate what a few-row product wants (one-off calls; loops pass their own buffer)."""
    if isinstance(workspace, str):
        need = earn_linear_workspace_bytes(rows, k, n)
        workspace = torch.empty(need, dtype=torch.uint8, device=device) if need else None
    return workspace, (0 if workspace is None else workspace.numel() * workspace.element_size())


def earn_qkv_rope_project(desc: AttnDesc, x, w_qkv, cu_seqlens, positions, batch: int, q_out, k_out, v_out,
                          workspace="auto") -> None:
    """w_qkv: [(Hq + 2 Hkv) d, d_model], outputs x inputs (the layout of a torch.nn.Linear weight)."""
    rows, d_model = x.shape
    n = (desc.n_q_heads + 2 * desc.n_kv_heads) * desc.head_dim
    assert tuple(w_qkv.shape) == (n, d_model)
    workspace, ws_bytes = _linear_workspace(rows, d_model, n, workspace, x.device)
    _check(lib().earn_qkv_rope_project(ctypes.byref(desc), _ptr(x), _ptr(w_qkv), rows, d_model, _ptr(cu_seqlens),
                                       _ptr(positions), batch, _ptr(q_out), _ptr(k_out), _ptr(v_out), _ptr(workspace),
                                       ws_bytes, _stream()))


def earn_linear(x, w, out, activation: int = 0, workspace="auto") -> None:
    """w: [n, k], outputs x inputs (the layout of a torch.nn.Linear weight)."""
    rows, k = x.shape
    n = w.shape[0]
    assert w.shape[1] == k and tuple(out.shape) == (rows, n)
    workspace, ws_bytes = _linear_workspace(rows, k, n, workspace, x.device)
    _check(lib().earn_linear(_ptr(x), _ptr(w), rows, k, n, activation, _ptr(out), _ptr(workspace), ws_bytes, _stream()))


def earn_attn_backward(desc: AttnDesc, q, k, v, out, lse, d_out, cu_seqlens, batch: int, total_tokens: int,
                       max_seqlen: int, dq, dk, dv, workspace=None) -> None:
    if workspace is None:
        need = int(lib().earn_attn_backward_workspace_bytes(ctypes.byref(desc), total_tokens))
        workspace = torch.empty(max(need, 1), dtype=torch.uint8, device=q.device)
    ws_bytes = workspace.numel() * workspace.element_size()
    _check(lib().earn_attn_backward(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), _ptr(d_out),
                                    _ptr(cu_seqlens), batch, total_tokens, max_seqlen, _ptr(dq), _ptr(dk), _ptr(dv),
                                    _ptr(workspace), ws_bytes, _stream()))


def _layer_stride(t: Optional[torch.Tensor]) -> int:
    """Bytes from one layer to the next of a [layers, ...] tensor (its layers must be contiguous blocks)."""
    if t is None:
        return 0
    assert t.is_cuda and t[0].is_contiguous(), "every layer of a layer-batched tensor must be contiguous"
    return t.stride(0) * t.element_size()


def earn_decode_layers_workspace_bytes(desc: AttnDesc, n_layers: int, n_streams: int, batch: int, max_shared_len: int,
                                       gen_cap: int) -> int:
    return int(lib().earn_decode_layers_workspace_bytes(ctypes.byref(desc), n_layers, n_streams, batch, max_shared_len,
                                                        gen_cap))


def _layers_ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def bind_prefill_attn_layers(desc: AttnDesc, q, k, v, cu_seqlens, positions, batch: int, total_tokens: int,
                             max_seqlen: int, out, k_rot_out, lse_out, workspace) -> BoundCall:
    """earn_prefill_attn_layers over [layers, tokens, heads, d] tensors (q, k, v, out, k_rot_out; lse_out
    [layers, tokens, Hq] or None), marshalled once; the layer strides are the tensors' own."""
    n_layers = q.shape[0]
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    args = (ctypes.byref(desc), n_layers, _layers_ptr(q), _layer_stride(q), _layers_ptr(k), _layers_ptr(v),
            _layer_stride(k), _ptr(cu_seqlens), _ptr(positions), batch, total_tokens, max_seqlen, _layers_ptr(out),
            _layer_stride(out), _layers_ptr(k_rot_out), _layer_stride(k_rot_out), _layers_ptr(lse_out),
            _layer_stride(lse_out), _ptr(workspace), ws_bytes)
    assert _layer_stride(k) == _layer_stride(v)
    return BoundCall(lib().earn_prefill_attn_layers, args, (desc, q, k, v, cu_seqlens, positions, out, k_rot_out, lse_out,
                                                            workspace))


def earn_prefill_attn_layers(desc: AttnDesc, q, k, v, cu_seqlens, positions, batch: int, total_tokens: int,
                             max_seqlen: int, out, k_rot_out, lse_out=None, workspace=None) -> None:
    if workspace is None:
        need = earn_prefill_workspace_bytes(desc, batch, total_tokens, max_seqlen, True)
        workspace = torch.empty(max(need, 1), dtype=torch.uint8, device=q.device)
    bind_prefill_attn_layers(desc, q, k, v, cu_seqlens, positions, batch, total_tokens, max_seqlen, out, k_rot_out,
                             lse_out, workspace)()


def bind_decode_attn_layers(desc: AttnDesc, q, k_new, v_new, q_pos, shared_k, shared_v, shared_cu, stream_to_seq, gen_k,
                            gen_v, gen_len, gen_cap: int, n_streams: int, batch: int, max_shared_len: int, out,
                            workspace) -> BoundCall:
    """earn_decode_attn_layers over [layers, ...] tensors (q, k_new, v_new, shared_k, shared_v, gen_k, gen_v, out),
    marshalled once; the layer strides are the tensors' own."""
    n_layers = q.shape[0]
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    assert _layer_stride(k_new) == _layer_stride(v_new) and _layer_stride(shared_k) == _layer_stride(shared_v)
    assert _layer_stride(gen_k) == _layer_stride(gen_v)
    args = (ctypes.byref(desc), n_layers, _layers_ptr(q), _layer_stride(q), _layers_ptr(k_new), _layers_ptr(v_new),
            _layer_stride(k_new), _ptr(q_pos), _layers_ptr(shared_k), _layers_ptr(shared_v), _layer_stride(shared_k),
            _ptr(shared_cu), _ptr(stream_to_seq), _layers_ptr(gen_k), _layers_ptr(gen_v), _layer_stride(gen_k),
            _ptr(gen_len), gen_cap, n_streams, batch, max_shared_len, _rows(shared_k, 1), _layers_ptr(out),
            _layer_stride(out), _ptr(workspace), ws_bytes)
    return BoundCall(lib().earn_decode_attn_layers, args, (desc, q, k_new, v_new, q_pos, shared_k, shared_v, shared_cu,
                                                           stream_to_seq, gen_k, gen_v, gen_len, out, workspace))


def earn_decode_attn_layers(desc: AttnDesc, q, k_new, v_new, q_pos, shared_k, shared_v, shared_cu, stream_to_seq, gen_k,
                            gen_v, gen_len, gen_cap: int, n_streams: int, batch: int, max_shared_len: int, out,
                            workspace=None) -> None:
    if workspace is None:
        need = earn_decode_layers_workspace_bytes(desc, q.shape[0], n_streams, batch, max_shared_len, gen_cap)
        workspace = torch.empty(max(need, 1), dtype=torch.uint8, device=q.device)
    bind_decode_attn_layers(desc, q, k_new, v_new, q_pos, shared_k, shared_v, shared_cu, stream_to_seq, gen_k, gen_v,
                            gen_len, gen_cap, n_streams, batch, max_shared_len, out, workspace)()


def earn_cache_entries(n_layers: int, split_k: int, seq_len: int, n_registers: int, gen: int = 0) -> int:
    return int(lib().earn_cache_entries(n_layers, split_k, seq_len, n_registers, gen))
