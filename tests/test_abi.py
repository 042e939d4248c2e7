"""The C-ABI library loads, exports every symbol include/earn.h declares, and rejects bad arguments on the host
(no kernel is launched by any call in this file, so it runs without a GPU)."""
import ctypes
import os
import re

import pytest

from paper_2507_00715_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "earn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(earn_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    names = declared_functions()
    assert set(names) == set(B.EXPORTS)
    lib = B.lib()
    for n in names:
        assert getattr(lib, n) is not None
    assert b"gfx950" in lib.earn_version()


def test_cache_entries_closed_form():
    # Section 3.3 typical values: k L + (N-k) r = 8*512 + 24*2
    assert B.earn_cache_entries(32, 8, 512, 2, 0) == 4144
    assert B.earn_cache_entries(4, 2, 100, 4, 4) == 2 * 100 + 2 * 4 + 4 * 4


def _desc(dtype=B.EARN_BF16, hq=4, hkv=2, d=64):
    return B.AttnDesc(dtype, hq, hkv, d, None, 0.0, 10000.0)


def test_prefill_argument_errors():
    lib = B.lib()
    fake = ctypes.c_void_p(256)  # never dereferenced: validation fails first
    call = lambda desc, q=fake, cu=fake, batch=1, total=8, maxlen=8, ws=0: lib.earn_prefill_attn(
        ctypes.byref(desc), q, fake, fake, cu, None, batch, total, maxlen, fake, fake, None, None, ws, None)
    assert call(_desc(d=96)) == B.EARN_ERR_UNSUPPORTED and b"head_dim" in lib.earn_last_error()
    assert call(_desc(dtype=7)) == B.EARN_ERR_UNSUPPORTED
    assert call(_desc(hq=5, hkv=2)) == B.EARN_ERR_INVALID_ARG and b"multiple" in lib.earn_last_error()
    assert call(_desc(), batch=0) == B.EARN_ERR_INVALID_ARG
    assert call(_desc(), q=None) == B.EARN_ERR_INVALID_ARG
    assert call(_desc(), cu=None) == B.EARN_ERR_INVALID_ARG
    assert call(_desc(), total=0) == B.EARN_OK          # empty batch is a no-op
    assert lib.earn_prefill_attn(None, fake, fake, fake, fake, None, 1, 8, 8, fake, None, None, None, 0, None) == B.EARN_ERR_INVALID_ARG
    # without k_rot_out the rotated keys need workspace
    rc = lib.earn_prefill_attn(ctypes.byref(_desc()), fake, fake, fake, fake, None, 1, 8, 8, fake, None, None, None, 0, None)
    assert rc == B.EARN_ERR_WORKSPACE_TOO_SMALL
    with_k = B.earn_prefill_workspace_bytes(_desc(), 1, 8, 8, True)      # bf16: the cos/sin table of the 8 tokens
    without_k = B.earn_prefill_workspace_bytes(_desc(), 1, 8, 8, False)  # plus the rotated keys
    assert with_k >= 8 * 32 * 8 and with_k % 256 == 0
    assert without_k - with_k >= 8 * 2 * 64 * 2 and without_k % 256 == 0
    # with k_rot_out but no workspace the bf16 path still lacks room for its table; the fp32 path needs none
    rc = lib.earn_prefill_attn(ctypes.byref(_desc()), fake, fake, fake, fake, None, 1, 8, 8, fake, fake, None, None, 0, None)
    assert rc == B.EARN_ERR_WORKSPACE_TOO_SMALL
    # one sequence's K/V rows are addressed with 32-bit byte offsets in the bf16 kernels
    big = 1 << 23  # 8 Mi tokens x 2 kv heads x 64 x 2 bytes = 2 GiB
    rc = lib.earn_prefill_attn(ctypes.byref(_desc()), fake, fake, fake, fake, None, 1, big, big, fake, fake, None, fake,
                               1 << 40, None)
    assert rc == B.EARN_ERR_UNSUPPORTED and b"2 GiB" in lib.earn_last_error()
    assert B.earn_prefill_workspace_bytes(_desc(dtype=B.EARN_F32), 1, 8, 8, True) == 0


def test_compact_argument_errors():
    lib = B.lib()
    fake = ctypes.c_void_p(256)
    vp = ctypes.c_void_p

    def call(n=1, src=256, dst=512, rb=32, cu=fake, batch=2, h=1, t=1):
        s, d, r = (vp * 1)(src), (vp * 1)(dst), (ctypes.c_int64 * 1)(rb)
        return lib.earn_compact_registers(n, s, d, r, cu, batch, 1024, h, t, None, None, None, None)

    assert call(batch=0) == B.EARN_ERR_INVALID_ARG
    assert call(h=0, t=0) == B.EARN_ERR_INVALID_ARG
    assert call(h=-1) == B.EARN_ERR_INVALID_ARG
    assert call(rb=24) == B.EARN_ERR_INVALID_ARG and b"multiple of 16" in lib.earn_last_error()
    assert call(rb=0) == B.EARN_ERR_INVALID_ARG
    assert call(src=264) == B.EARN_ERR_INVALID_ARG and b"aligned" in lib.earn_last_error()
    assert call(src=None) == B.EARN_ERR_INVALID_ARG
    assert call(cu=None) == B.EARN_ERR_INVALID_ARG
    assert call(n=B.EARN_MAX_COMPACT_TENSORS + 1) == B.EARN_ERR_INVALID_ARG
    assert lib.earn_compact_registers(1, None, None, None, fake, 2, 1024, 1, 1, None, None, None, None) == B.EARN_ERR_INVALID_ARG


def test_decode_argument_errors():
    lib = B.lib()
    fake = ctypes.c_void_p(256)

    def call(desc=None, q=fake, s2s=fake, gen_cap=4, S=2, batch=2, maxlen=8, ws=None, ws_bytes=0):
        desc = desc or _desc()
        return lib.earn_decode_attn(ctypes.byref(desc), q, fake, fake, fake, fake, fake, fake, s2s, fake, fake, fake,
                                    gen_cap, S, batch, maxlen, 1 << 20, fake, ws, ws_bytes, None)

    assert call(desc=_desc(d=32)) == B.EARN_ERR_UNSUPPORTED
    assert call(q=None) == B.EARN_ERR_INVALID_ARG
    assert call(gen_cap=0) == B.EARN_ERR_INVALID_ARG
    assert call(S=0) == B.EARN_ERR_INVALID_ARG
    assert call(maxlen=-1) == B.EARN_ERR_INVALID_ARG
    assert call(s2s=None, S=4, batch=2) == B.EARN_ERR_INVALID_ARG and b"stream_to_seq" in lib.earn_last_error()
    # long caches are split over workgroups and need workspace for the partial results
    need = B.earn_decode_workspace_bytes(_desc(), 2, 2, 100000, 4)
    assert need > 0
    assert call(maxlen=100000) == B.EARN_ERR_WORKSPACE_TOO_SMALL
    assert B.earn_decode_workspace_bytes(_desc(hq=64, hkv=64), 512, 512, 16, 4) == 0
    # limits of the matrix-core kernel: beams per sequence, query heads per kv head
    assert call(S=1500, batch=1, maxlen=500) == B.EARN_ERR_UNSUPPORTED and b"streams" in lib.earn_last_error()
    assert call(desc=_desc(hq=32, hkv=2, d=64)) == B.EARN_ERR_UNSUPPORTED and b"query heads" in lib.earn_last_error()
    # many sequences: the key range of the matrix-core kernel is not split either, no partial results
    assert B.earn_decode_workspace_bytes(_desc(hq=12, hkv=2, d=128), 256, 256, 1038, 4) == 0
    # few sequences with long caches: one partial (d + 2 floats) per (stream, head, split), at least two splits
    assert B.earn_decode_workspace_bytes(_desc(hq=32, hkv=8, d=128), 160, 16, 8256, 8) >= 2 * 160 * 32 * (128 + 2) * 4


def test_register_rows_argument_errors():
    lib = B.lib()
    fake = ctypes.c_void_p(256)

    def call(desc=None, q=fake, pos=fake, batch=2, total=600, maxlen=400, r=8, krot=fake, ws=None, ws_bytes=0):
        desc = desc or _desc(hq=8, hkv=2, d=128)
        return lib.earn_prefill_register_rows(ctypes.byref(desc), q, fake, fake, fake, pos, batch, total, maxlen, r,
                                              fake, krot, ws, ws_bytes, None)

    assert call(q=None) == B.EARN_ERR_INVALID_ARG
    assert call(pos=None) == B.EARN_ERR_INVALID_ARG
    assert call(krot=None) == B.EARN_ERR_INVALID_ARG          # the rotated keys are the layer's cache: required
    assert call(batch=0) == B.EARN_ERR_INVALID_ARG
    assert call(r=0) == B.EARN_ERR_INVALID_ARG
    assert call(r=500) == B.EARN_ERR_INVALID_ARG and b"rows_per_seq" in lib.earn_last_error()
    assert B.earn_prefill_register_rows_workspace_bytes(_desc(dtype=B.EARN_F32, hq=8, hkv=2, d=128), 2, 400, 8) == 0
    assert call(desc=_desc(hq=8, hkv=2, d=32)) == B.EARN_ERR_UNSUPPORTED
    # two sequences x two kv heads leave room for key splits: partial results need workspace
    need = B.earn_prefill_register_rows_workspace_bytes(_desc(hq=8, hkv=2, d=128), 2, 400, 8)
    assert need >= 2 * (2 * 8) * 8 * (128 + 2) * 4 and need % 4 == 0
    assert call() == B.EARN_ERR_WORKSPACE_TOO_SMALL
    # enough (sequence, kv head) pairs: nothing is split, no workspace
    assert B.earn_prefill_register_rows_workspace_bytes(_desc(hq=8, hkv=8, d=128), 64, 400, 8) == 0
    assert B.earn_prefill_register_rows_workspace_bytes(_desc(hq=8, hkv=3, d=128), 2, 400, 8) == 0  # invalid desc


def test_binding_refuses_host_tensors():
    import torch
    with pytest.raises(AssertionError):
        B.earn_compact_registers([torch.zeros(4, 16, dtype=torch.uint8)], [torch.zeros(2, 16, dtype=torch.uint8)],
                                 torch.zeros(2, dtype=torch.int32), 1, 1, 1)
