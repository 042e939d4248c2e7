"""Seeded synthetic workloads for the EARN attention hot path.

This module only *draws inputs*: sequence lengths, the packed ragged layout
X = [R_prefix; Prompt; R_suffix] (paper Eq. 5) and N(0,1) tensors for Q/K/V.
It holds none of the method's arithmetic (no RoPE, no softmax, no gather), so
both the CPU oracle and the HIP path may be fed from it.

Every value is a pure function of integer coordinates:

    value(stream_key, seq, pos, col) = NORMAL_TABLE[ mix64(stream_key ^ pack(seq, pos, col)) >> 48 ]

mix64 is the splitmix64 finaliser in wrapping 64-bit integer arithmetic and
NORMAL_TABLE holds the 65536 mid-point quantiles of N(0,1).  Only integer ops
and one table lookup are involved, so the CPU and the GPU produce bit-identical
tensors, and any row can be drawn without materialising the whole tensor
(needed for sampled checks at the large configurations).

The five configurations are the ones the benchmark definition names; the
paper's datasets are not available, so these stand in for its workloads with
the paper's shapes (Section 3.3 "typical values", Section 4.1 backbones,
Appendix A.3 identifier length and beam search).
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

BASE_SEED = 250700715

_M64 = (1 << 64) - 1
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB
_GOLD = 0x9E3779B97F4A7C15

# tensor ids (field of the stream key)
T_Q, T_K, T_V, T_X, T_DQ, T_DK, T_DV, T_LEN, T_OUTLIER = range(1, 10)


def _signed(c: int) -> int:
    c &= _M64
    return c - (1 << 64) if c >= (1 << 63) else c


def mix64_int(z: int) -> int:
    """splitmix64 finaliser on a Python int (reference for the tensor version)."""
    z &= _M64
    z = ((z ^ (z >> 30)) * _C1) & _M64
    z = ((z ^ (z >> 27)) * _C2) & _M64
    return z ^ (z >> 31)


def stream_key(seed: int, config_id: int, layer: int, tensor_id: int, extra: int = 0) -> int:
    """Fold the identifying fields of one tensor into a 64-bit key (host side)."""
    z = mix64_int(seed * _GOLD + 1)
    for f in (config_id, layer, tensor_id, extra):
        z = mix64_int(z ^ ((f + 1) * _GOLD))
    return z


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix64(z: torch.Tensor) -> torch.Tensor:
    z = (z ^ _lsr(z, 30)) * _signed(_C1)
    z = (z ^ _lsr(z, 27)) * _signed(_C2)
    return z ^ _lsr(z, 31)


_TABLE_CACHE: Dict[str, torch.Tensor] = {}


def normal_table(device="cpu") -> torch.Tensor:
    """65536 mid-point quantiles of N(0,1) in fp32 (computed once, in fp64, on the host)."""
    dev = str(torch.device(device))
    if "cpu" not in _TABLE_CACHE:
        from scipy.special import ndtri

        u = (np.arange(65536, dtype=np.float64) + 0.5) / 65536.0
        _TABLE_CACHE["cpu"] = torch.from_numpy(ndtri(u).astype(np.float32))
    if dev not in _TABLE_CACHE:
        _TABLE_CACHE[dev] = _TABLE_CACHE["cpu"].to(dev)
    return _TABLE_CACHE[dev]


def _hash16(key: int, seq: torch.Tensor, pos: torch.Tensor, ncols: int) -> torch.Tensor:
    """[rows, ncols] int64 in [0, 65536) for rows given by (seq, pos)."""
    dev = seq.device
    col = torch.arange(ncols, dtype=torch.int64, device=dev)
    row = (seq.to(torch.int64) << 40) | (pos.to(torch.int64) << 20)
    z = (row[:, None] | col[None, :]) ^ _signed(key)
    return _lsr(_mix64(z), 48)


def normal_rows(key: int, seq: torch.Tensor, pos: torch.Tensor, ncols: int,
                dtype: torch.dtype = torch.float32, chunk_rows: int = 1 << 15) -> torch.Tensor:
    """N(0,1) rows for coordinates (seq[i], pos[i]), shape [len(seq), ncols], on seq's device.

    seq < 2**23, pos < 2**20, ncols <= 2**20.
    """
    assert seq.shape == pos.shape and seq.dim() == 1
    assert ncols <= (1 << 20)
    table = normal_table(seq.device)
    out = torch.empty((seq.numel(), ncols), dtype=dtype, device=seq.device)
    for r0 in range(0, seq.numel(), chunk_rows):
        r1 = min(seq.numel(), r0 + chunk_rows)
        idx = _hash16(key, seq[r0:r1], pos[r0:r1], ncols)
        out[r0:r1] = table[idx].to(dtype)
    return out


def bernoulli_rows(key: int, seq: torch.Tensor, pos: torch.Tensor, ncols: int, prob: float) -> torch.Tensor:
    """[rows, ncols] bool, True with probability `prob` (same counter scheme)."""
    thr = int(round(prob * 65536.0))
    return _hash16(key, seq, pos, ncols) < thr


def uniform_ints(key: int, count: int, lo: int, hi: int) -> List[int]:
    """`count` integers uniform on [lo, hi] (host side, exact integer arithmetic)."""
    return [lo + mix64_int(key ^ ((i + 1) * _GOLD)) % (hi - lo + 1) for i in range(count)]


def log_uniform_ints(key: int, count: int, lo: int, hi: int) -> List[int]:
    """`count` integers with log-uniform density on [lo, hi] (host side)."""
    out = []
    for i in range(count):
        u = (mix64_int(key ^ ((i + 1) * _GOLD)) >> 11) / float(1 << 53)
        out.append(min(hi, int(math.floor(math.exp(math.log(lo) + u * (math.log(hi + 1) - math.log(lo)))))))
    return out


# --------------------------------------------------------------------------------------
# configurations
# --------------------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class Config:
    name: str
    config_id: int
    dtype: str               # "f32" | "bf16"
    batch: int
    len_dist: tuple          # ("list", [..]) | ("uniform", lo, hi) | ("loguniform", lo, hi) | ("fixed", L)
    n_head_reg: int          # h
    n_tail_reg: int          # t
    n_layers: int            # N
    split_k: int             # k
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    decode_steps: int        # G
    beams: int = 1           # W
    outlier_prob: float = 0.0
    outlier_scale: float = 8.0
    rope_base: float = 10000.0

    @property
    def r(self) -> int:
        return self.n_head_reg + self.n_tail_reg

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def replace(self, **kw) -> "Config":
        return dataclasses.replace(self, **kw)


CONFIGS: Dict[str, Config] = {
    "tiny_f32": Config("tiny_f32", 1, "f32", 2, ("list", (96, 128)), 2, 2, 4, 2, 4, 4, 64, 4),
    "small_gqa": Config("small_gqa", 2, "bf16", 32, ("uniform", 256, 512), 8, 8, 24, 4, 14, 2, 64, 16),
    "mid_mha": Config("mid_mha", 3, "bf16", 64, ("uniform", 256, 2048), 16, 16, 32, 8, 32, 32, 128, 8,
                      outlier_prob=0.05),
    "long_beam": Config("long_beam", 4, "bf16", 16, ("fixed", 8192), 32, 32, 32, 4, 32, 8, 128, 8, beams=10),
    "serving": Config("serving", 5, "bf16", 256, ("loguniform", 64, 1024), 8, 8, 28, 2, 12, 2, 128, 4),
    # Prefill-only workload in the shape of a sequential-recommendation transducer of the HSTU kind (the paper's
    # appendix instantiates EARN on HSTU: item-id histories, no prompt text, one output embedding, hence no decode
    # stage; it reports about 2x speedup and 50 % memory savings there, i.e. k = N/2): 128 user histories of 256-4096
    # actions, 8 heads of 128, 16 layers split at 8, 4 + 4 registers.  Softmax attention stands in for that model's
    # pointwise attention: the shapes, not the activation, are what this path exercises.
    "hstu_prefill": Config("hstu_prefill", 6, "bf16", 128, ("loguniform", 256, 4096), 4, 4, 16, 8, 8, 8, 128, 0),
}
CONFIG_ORDER = ["tiny_f32", "small_gqa", "mid_mha", "long_beam", "serving", "hstu_prefill"]


class Workload:
    """Lengths and layout of one configuration plus on-demand tensor draws."""

    def __init__(self, cfg: Config, seed: int = BASE_SEED, history_lengths: Optional[Sequence[int]] = None):
        self.cfg = cfg
        self.seed = seed
        if history_lengths is None:
            kind = cfg.len_dist[0]
            lkey = stream_key(seed, cfg.config_id, 0, T_LEN)
            if kind == "list":
                history_lengths = list(cfg.len_dist[1])
            elif kind == "fixed":
                history_lengths = [cfg.len_dist[1]] * cfg.batch
            elif kind == "uniform":
                history_lengths = uniform_ints(lkey, cfg.batch, cfg.len_dist[1], cfg.len_dist[2])
            elif kind == "loguniform":
                history_lengths = log_uniform_ints(lkey, cfg.batch, cfg.len_dist[1], cfg.len_dist[2])
            else:
                raise ValueError(kind)
        assert len(history_lengths) == cfg.batch
        self.history_lengths = [int(x) for x in history_lengths]          # L_s
        self.seq_lengths = [cfg.r + L for L in self.history_lengths]       # n_s = h + L_s + t
        cu = [0]
        for n in self.seq_lengths:
            cu.append(cu[-1] + n)
        self.cu_seqlens = cu
        self.total_tokens = cu[-1]
        self.max_seqlen = max(self.seq_lengths)
        self.n_streams = cfg.batch * cfg.beams
        self.stream_to_seq = [u // cfg.beams for u in range(self.n_streams)]

    # ---- coordinates ----
    def token_coords(self, device="cpu", seqs: Optional[Sequence[int]] = None):
        """(seq, pos) int64 vectors for the packed tokens of `seqs` (default: all sequences)."""
        seqs = range(self.cfg.batch) if seqs is None else seqs
        lens = torch.tensor([self.seq_lengths[s] for s in seqs], dtype=torch.int64, device=device)
        sid = torch.tensor(list(seqs), dtype=torch.int64, device=device)
        seq = torch.repeat_interleave(sid, lens)
        start = torch.cumsum(lens, 0) - lens
        pos = torch.arange(int(lens.sum()), dtype=torch.int64, device=device) - torch.repeat_interleave(start, lens)
        return seq, pos

    def _key(self, layer: int, tensor_id: int, extra: int = 0) -> int:
        return stream_key(self.seed, self.cfg.config_id, layer, tensor_id, extra)

    # ---- prefill tensors ----
    def prefill_tensor(self, which: str, layer: int, device="cpu", seqs=None, heads: Optional[Sequence[int]] = None,
                       coords=None) -> torch.Tensor:
        """Q ('q'), K ('k'), V ('v') of one layer as [tokens, heads, d], or the hidden stand-in 'x' as [tokens, Hq*d].

        `seqs` restricts to some sequences (packed in that order), `heads` to some heads, and
        `coords=(seq, pos)` to arbitrary tokens; the values do not depend on the restriction.
        """
        cfg = self.cfg
        tid = {"q": T_Q, "k": T_K, "v": T_V, "x": T_X}[which]
        H = cfg.n_q_heads if which in ("q", "x") else cfg.n_kv_heads
        ncols = H * cfg.head_dim
        seq, pos = coords if coords is not None else self.token_coords(device, seqs)
        t = normal_rows(self._key(layer, tid), seq, pos, ncols, cfg.torch_dtype)
        if which == "x":
            return t
        t = t.view(-1, H, cfg.head_dim)
        if which == "k" and cfg.outlier_prob > 0.0:
            mask = bernoulli_rows(self._key(layer, T_OUTLIER), seq, pos, H, cfg.outlier_prob)
            t = torch.where(mask[:, :, None], t * cfg.outlier_scale, t)
        if heads is not None:
            t = t[:, list(heads), :].contiguous()
        return t

    # ---- decode tensors ----
    def decode_tensor(self, which: str, layer: int, step: int, device="cpu",
                      streams: Optional[Sequence[int]] = None) -> torch.Tensor:
        """q ('q') [S,Hq,d] or k_new/v_new ('k'/'v') [S,Hkv,d] of decode step `step`."""
        cfg = self.cfg
        tid = {"q": T_DQ, "k": T_DK, "v": T_DV}[which]
        H = cfg.n_q_heads if which == "q" else cfg.n_kv_heads
        streams = range(self.n_streams) if streams is None else streams
        sid = torch.tensor(list(streams), dtype=torch.int64, device=device)
        pos = torch.full_like(sid, step)
        t = normal_rows(self._key(layer, tid), sid, pos, H * cfg.head_dim, cfg.torch_dtype)
        return t.view(-1, H, cfg.head_dim)

    def decode_positions(self, step: int) -> List[int]:
        """Original position of the token generated at `step` for every stream: n_s + step."""
        return [self.seq_lengths[self.stream_to_seq[u]] + step for u in range(self.n_streams)]

    # ---- bookkeeping the harness prints ----
    def causal_pairs(self, compacted: bool = False) -> int:
        if compacted:
            return self.cfg.batch * self.cfg.r * (self.cfg.r + 1) // 2
        return sum(n * (n + 1) // 2 for n in self.seq_lengths)

    def describe(self) -> dict:
        c = self.cfg
        return {"workload": c.name, "dtype": c.dtype, "batch": c.batch, "total_tokens": self.total_tokens,
                "min_len": min(self.seq_lengths), "max_len": self.max_seqlen, "head_regs": c.n_head_reg,
                "tail_regs": c.n_tail_reg, "layers": c.n_layers, "split_k": c.split_k, "q_heads": c.n_q_heads,
                "kv_heads": c.n_kv_heads, "head_dim": c.head_dim, "decode_steps": c.decode_steps, "beams": c.beams,
                "seed": self.seed, "seq_lengths": list(self.seq_lengths)}


def to_f64(t: torch.Tensor) -> np.ndarray:
    """Exact widening of an fp32/bf16 tensor to a contiguous fp64 numpy array."""
    return t.detach().to("cpu").to(torch.float64).contiguous().numpy()
