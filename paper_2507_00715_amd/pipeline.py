"""The EARN attention path on the GPU, expressed as calls into libearn (paper Section 3.2, Inference).

    first k layers   earn_prefill_attn on all tokens; the rotated keys and the values are the layer's cache
    layer k input    earn_compact_registers gathers the register rows (hidden-state stand-in and the per-layer
                     Q/K/V of the remaining layers, which in a full model would be projected from the gathered rows)
    layers k..N-1    earn_prefill_attn on the r = h+t register rows with their original positions
    decode step g    earn_decode_attn per layer: full cache for layers < k, register cache for layers >= k

With rows_only_last_full_layer=True, layer k-1 — whose outputs at prompt tokens nothing downstream reads, since the
input of layer k keeps the register rows only — is evaluated at the register rows alone (earn_prefill_register_rows on
the gathered query rows); its keys and values stay full length, they are the layer's cache.  prefill_out[k-1] then
holds the B*r register rows in compacted order.

Per-layer buffers of one kind are slices of ONE tensor with a leading layer dimension (register layers k..N-1: gathered
q/k/v, caches, outputs; full layers 0..k-1: key caches, decode outputs; generated caches of all layers), so that the
layer-batched entry points (earn_prefill_attn_layers, earn_decode_attn_layers) can take a run of layers in one launch
when the layers are independent of each other, as they are with synthetic per-layer inputs; the per-layer methods work
on the same slices.

All buffers are allocated once in the constructor; the methods only enqueue kernels on the current stream.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import torch

from . import binding as B


def capture_graph(calls) -> "torch.cuda.CUDAGraph":
    """Record a sequence of launches into a HIP graph and return it; `replay()` then enqueues the whole sequence with
    one call.  For the launch-bound stretches of the path in the form a real model needs them (layer l+1 reads what
    layer l wrote, so the layers cannot share a launch): a decode step is N small launches per step, each costing more
    host time than GPU time.  `calls` are objects that only enqueue kernels on the current stream on buffers that stay
    where they are (BoundCall objects, or the path's methods with fixed arguments): the entry points allocate nothing
    and do not synchronise, and none of them clears memory with a memset node.  The validation mode (which copies to
    the host) must be off."""
    side = torch.cuda.Stream()                       # default priority
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                    # one eager pass first: nothing lazy is left for the capture
        for c in calls:
            c()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for c in calls:
            c()
    return graph


class EarnPath:
    def __init__(self, *, n_layers: int, split_k: int, n_head_reg: int, n_tail_reg: int, n_q_heads: int,
                 n_kv_heads: int, head_dim: int, dtype: torch.dtype, cu_seqlens: Sequence[int],
                 stream_to_seq: Sequence[int], gen_cap: int, rope_base: float = 10000.0, softmax_scale: float = 0.0,
                 device="cuda:0", want_lse: bool = False, rows_only_last_full_layer: bool = False):
        self.N, self.k, self.h, self.t = n_layers, split_k, n_head_reg, n_tail_reg
        self.r = n_head_reg + n_tail_reg
        self.hq, self.hkv, self.d, self.dtype = n_q_heads, n_kv_heads, head_dim, dtype
        self.device = torch.device(device)
        self.desc = B.make_desc(dtype, n_q_heads, n_kv_heads, head_dim, softmax_scale, rope_base)
        lens = [cu_seqlens[i + 1] - cu_seqlens[i] for i in range(len(cu_seqlens) - 1)]
        self.lens = lens
        self.batch = len(lens)
        self.T = int(cu_seqlens[-1])
        self.max_seqlen = max(lens)
        self.Tc = self.batch * self.r
        self.S = len(stream_to_seq)
        self.gen_cap = gen_cap
        self.rows_only = bool(rows_only_last_full_layer) and 0 < split_k < n_layers
        dev, i32 = self.device, torch.int32
        self.cu = torch.tensor(list(cu_seqlens), dtype=i32, device=dev)
        # one stream per sequence in order: the library takes "no map" and saves every decode workgroup a dependent load
        identity = list(stream_to_seq) == list(range(self.batch))
        self.stream_to_seq = None if identity else torch.tensor(list(stream_to_seq), dtype=i32, device=dev)
        # written by the compaction; valid (if not yet meaningful) before it has run, so that a call bound to them can be
        # launched at any time: the library trusts cu_seqlens arrays
        self.idx = torch.zeros(self.Tc, dtype=i32, device=dev)
        self.pos = torch.zeros(self.Tc, dtype=i32, device=dev)
        self.cu_c = torch.arange(0, (self.batch + 1) * self.r, self.r, dtype=i32, device=dev)
        e = lambda *shape: torch.empty(shape, dtype=dtype, device=dev)
        N, k = self.N, self.k
        rows_layer = k - 1 if self.rows_only else -1
        R = N - k                                                     # register-focused layers
        # stacks with a leading layer dimension; the per-layer lists below are slices of them
        self.reg_prefill_out = e(R, self.Tc, self.hq, self.d)
        self.reg_q, self.reg_k, self.reg_v = e(R, self.Tc, self.hq, self.d), e(R, self.Tc, self.hkv, self.d), e(R, self.Tc, self.hkv, self.d)
        self.reg_k_cache = e(R, self.Tc, self.hkv, self.d)
        self.full_k_cache = e(k, self.T, self.hkv, self.d)
        self.gen_k_all = torch.zeros(N, self.S, gen_cap, self.hkv, self.d, dtype=dtype, device=dev)
        self.gen_v_all = torch.zeros(N, self.S, gen_cap, self.hkv, self.d, dtype=dtype, device=dev)
        self.decode_out_all = e(N, self.S, self.hq, self.d)
        self.prefill_out = [(e(self.T, self.hq, self.d) if l != rows_layer else e(self.Tc, self.hq, self.d)) if l < k
                            else self.reg_prefill_out[l - k] for l in range(N)]
        self.q_rows = e(self.Tc, self.hq, self.d) if self.rows_only else None
        self.k_cache = [self.full_k_cache[l] if l < k else self.reg_k_cache[l - k] for l in range(N)]
        self.v_cache: List[Optional[torch.Tensor]] = [None] * N       # layers < k alias the caller's V
        self.v_full_stack: Optional[torch.Tensor] = None              # [k, T, Hkv, d], if the caller keeps V that way
        self.x_c: Optional[torch.Tensor] = None
        self.q_c = {l: self.reg_q[l - k] for l in range(k, N)}
        self.k_c = {l: self.reg_k[l - k] for l in range(k, N)}
        self.v_c = {l: self.reg_v[l - k] for l in range(k, N)}
        self.reg_lse = torch.empty(R, self.Tc, self.hq, dtype=torch.float32, device=dev) if want_lse else None
        self.lse = ([torch.empty(self.T, self.hq, dtype=torch.float32, device=dev) if l < k else self.reg_lse[l - k]
                     for l in range(N)] if want_lse else [None] * N)
        self.gen_k = [self.gen_k_all[l] for l in range(N)]
        self.gen_v = [self.gen_v_all[l] for l in range(N)]
        self.gen_len = torch.zeros(self.S, dtype=i32, device=dev)
        self.q_pos = torch.zeros(self.S, dtype=i32, device=dev)
        self.decode_out = [self.decode_out_all[l] for l in range(N)]
        ws = max(B.earn_decode_workspace_bytes(self.desc, self.S, self.batch, self.max_seqlen, gen_cap),
                 B.earn_decode_workspace_bytes(self.desc, self.S, self.batch, self.r, gen_cap),
                 B.earn_decode_layers_workspace_bytes(self.desc, max(k, 1), self.S, self.batch, self.max_seqlen, gen_cap),
                 B.earn_decode_layers_workspace_bytes(self.desc, max(R, 1), self.S, self.batch, self.r, gen_cap), 256)
        self.workspace = torch.empty(ws, dtype=torch.uint8, device=dev)
        pws = max(B.earn_prefill_workspace_bytes(self.desc, self.batch, self.T, self.max_seqlen, True),
                  B.earn_prefill_workspace_bytes(self.desc, self.batch, self.Tc, self.r, True), 256)
        if self.rows_only:
            pws = max(pws, B.earn_prefill_register_rows_workspace_bytes(self.desc, self.batch, self.max_seqlen, self.r))
        self.prefill_workspace = torch.empty(pws, dtype=torch.uint8, device=dev)

    # ---- prefill ----
    def prefill_full_layer(self, l: int, q, k, v) -> None:
        B.earn_prefill_attn(self.desc, q, k, v, self.cu, None, self.batch, self.T, self.max_seqlen,
                            self.prefill_out[l], self.k_cache[l], self.lse[l], self.prefill_workspace)
        self.v_cache[l] = v

    def prefill_last_full_layer_rows(self, q, k, v) -> None:
        """Layer k-1 at the register rows only: gather its query rows (which also yields idx/pos/cu_c), then attend."""
        l = self.k - 1
        B.earn_compact_registers([q], [self.q_rows], self.cu, self.batch, self.h, self.t, self.idx, self.pos, self.cu_c)
        B.earn_prefill_register_rows(self.desc, self.q_rows, k, v, self.cu, self.pos, self.batch, self.T,
                                     self.max_seqlen, self.r, self.prefill_out[l], self.k_cache[l],
                                     self.prefill_workspace)
        self.v_cache[l] = v

    def compact(self, x: Optional[torch.Tensor], q: Sequence[torch.Tensor], k: Sequence[torch.Tensor],
                v: Sequence[torch.Tensor]) -> None:
        """Gather register rows of x and of the per-layer q/k/v for layers k..N-1 (indexable by layer)."""
        src, dst = [], []
        if x is not None:
            if self.x_c is None or self.x_c.shape[1:] != x.shape[1:]:
                self.x_c = torch.empty((self.Tc,) + tuple(x.shape[1:]), dtype=x.dtype, device=self.device)
            src.append(x)
            dst.append(self.x_c)
        for l in range(self.k, self.N):
            src += [q[l], k[l], v[l]]
            dst += [self.q_c[l], self.k_c[l], self.v_c[l]]
        first = True
        for i in range(0, max(len(src), 1), B.EARN_MAX_COMPACT_TENSORS):
            B.earn_compact_registers(src[i:i + B.EARN_MAX_COMPACT_TENSORS], dst[i:i + B.EARN_MAX_COMPACT_TENSORS],
                                     self.cu, self.batch, self.h, self.t, self.idx if first else None,
                                     self.pos if first else None, self.cu_c if first else None)
            first = False

    def prefill_register_layer(self, l: int) -> None:
        B.earn_prefill_attn(self.desc, self.q_c[l], self.k_c[l], self.v_c[l], self.cu_c, self.pos, self.batch,
                            self.Tc, self.r, self.prefill_out[l], self.k_cache[l], self.lse[l], self.prefill_workspace)
        self.v_cache[l] = self.v_c[l]

    def prefill(self, q: Sequence[torch.Tensor], k: Sequence[torch.Tensor], v: Sequence[torch.Tensor],
                x: Optional[torch.Tensor]) -> None:
        for l in range(self.k):
            if self.rows_only and l == self.k - 1:
                self.prefill_last_full_layer_rows(q[l], k[l], v[l])
            else:
                self.prefill_full_layer(l, q[l], k[l], v[l])
        if self.k < self.N:
            self.compact(x, q, k, v)
            for l in range(self.k, self.N):
                self.prefill_register_layer(l)

    def bind_prefill_register_layers(self) -> "B.BoundCall":
        """All register-focused layers k..N-1 in one launch (valid when the layers' inputs do not depend on each other:
        the gathered q/k/v of the synthetic workloads), marshalled once."""
        for l in range(self.k, self.N):
            self.v_cache[l] = self.v_c[l]
        return B.bind_prefill_attn_layers(self.desc, self.reg_q, self.reg_k, self.reg_v, self.cu_c, self.pos, self.batch,
                                          self.Tc, self.r, self.reg_prefill_out, self.reg_k_cache, self.reg_lse,
                                          self.prefill_workspace)

    # ---- decode ----
    def set_step(self, g: int) -> None:
        """gen_len = g and q_pos = n_s + g for every stream (one small kernel of the library, no host sync)."""
        B.earn_decode_step_positions(self.cu, self.stream_to_seq, self.S, self.batch, g, self.q_pos, self.gen_len)

    def bind_set_step(self, g: int) -> "B.BoundCall":
        return B.bind_decode_step_positions(self.cu, self.stream_to_seq, self.S, self.batch, g, self.q_pos, self.gen_len)

    def bind_decode_register_layers(self, dq, dk, dv) -> "B.BoundCall":
        """One decode step of all register-focused layers in one launch; dq/dk/dv: [N-k, S, H, d]."""
        return B.bind_decode_attn_layers(self.desc, dq, dk, dv, self.q_pos, self.reg_k_cache, self.reg_v, self.cu_c,
                                         self.stream_to_seq, self.gen_k_all[self.k:], self.gen_v_all[self.k:],
                                         self.gen_len, self.gen_cap, self.S, self.batch, self.r,
                                         self.decode_out_all[self.k:], self.workspace)

    def bind_decode_full_layers(self, dq, dk, dv) -> "B.BoundCall":
        """One decode step of the first k layers in one launch; dq/dk/dv: [k, S, H, d]; needs v_full_stack [k, T, Hkv, d]
        (the values the prefill of those layers was given, kept as one tensor)."""
        assert self.v_full_stack is not None and self.v_full_stack.shape[0] == self.k
        return B.bind_decode_attn_layers(self.desc, dq, dk, dv, self.q_pos, self.full_k_cache, self.v_full_stack, self.cu,
                                         self.stream_to_seq, self.gen_k_all[:self.k], self.gen_v_all[:self.k],
                                         self.gen_len, self.gen_cap, self.S, self.batch, self.max_seqlen,
                                         self.decode_out_all[:self.k], self.workspace)

    def decode_layer(self, l: int, dq, dk, dv) -> None:
        full = l < self.k
        B.earn_decode_attn(self.desc, dq, dk, dv, self.q_pos, self.k_cache[l], self.v_cache[l],
                           self.cu if full else self.cu_c, self.stream_to_seq, self.gen_k[l], self.gen_v[l],
                           self.gen_len, self.gen_cap, self.S, self.batch, self.max_seqlen if full else self.r,
                           self.decode_out[l], self.workspace)

    def bind_decode_layer(self, l: int, dq, dk, dv) -> "B.BoundCall":
        """decode_layer(l, dq, dk, dv) with its arguments marshalled once: for loops that replay the same buffers."""
        full = l < self.k
        return B.bind_decode_attn(self.desc, dq, dk, dv, self.q_pos, self.k_cache[l], self.v_cache[l],
                                  self.cu if full else self.cu_c, self.stream_to_seq, self.gen_k[l], self.gen_v[l],
                                  self.gen_len, self.gen_cap, self.S, self.batch, self.max_seqlen if full else self.r,
                                  self.decode_out[l], self.workspace)

    def bind_prefill_register_layer(self, l: int) -> "B.BoundCall":
        """prefill_register_layer(l), marshalled once (valid after compact() has run once: v_cache[l] is set here)."""
        self.v_cache[l] = self.v_c[l]
        return B.bind_prefill_attn(self.desc, self.q_c[l], self.k_c[l], self.v_c[l], self.cu_c, self.pos, self.batch,
                                   self.Tc, self.r, self.prefill_out[l], self.k_cache[l], self.lse[l],
                                   self.prefill_workspace)

    def decode_step(self, g: int, dq: Sequence[torch.Tensor], dk: Sequence[torch.Tensor],
                    dv: Sequence[torch.Tensor]) -> None:
        self.set_step(g)
        for l in range(self.N):
            self.decode_layer(l, dq[l], dk[l], dv[l])
