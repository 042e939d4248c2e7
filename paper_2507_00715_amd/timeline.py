"""Where a workgroup of the medium-length bf16 prefill kernel spends its life.

`python -m paper_2507_00715_amd.timeline [workload]` compiles `csrc/prefill.hip` once more with `-DEARN_PF_TIMELINE`
(life-cycle timers in `prefill_mfma_kernel`, see the comment above that kernel), links it with the objects of the normal
build into `libearn_timeline.so` beside `libearn.so`, runs one full-length prefill layer of the workload through the
C ABI and prints what thread 0 of every workgroup stamped: the phases of a workgroup's life, the time between two
workgroups on one CU, and how many workgroups a CU holds at a time.  A diagnostic: nothing on the product path uses
the timeline library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import sys

import numpy as np
import torch

from . import build as earn_build

TIMELINE_LIB = os.path.join(earn_build.HERE, "libearn_timeline.so")
TICK_US = 0.01  # the wall clock of the device counts at 100 MHz


def build_timeline_library(force: bool = False) -> str:
    """Compile prefill.hip with the timers and link it with the normal build's other objects (built first if absent).
    Kept, unless `force`, when it is newer than every source."""
    sources = [os.path.join(earn_build.CSRC, f) for f in os.listdir(earn_build.CSRC) if f.endswith((".hip", ".h"))]
    if not force and os.path.exists(TIMELINE_LIB) and all(os.path.getmtime(TIMELINE_LIB) >= os.path.getmtime(f) for f in sources):
        return TIMELINE_LIB
    objs = [os.path.join(earn_build.CSRC, s.replace(".hip", ".o")) for s in earn_build.SOURCES]
    if not all(os.path.exists(o) and os.path.getmtime(o) >= max(os.path.getmtime(f) for f in sources) for o in objs):
        earn_build.build(verbose=False)
    obj = os.path.join(earn_build.CSRC, "prefill_timeline.o")
    r = subprocess.run(["hipcc", *earn_build.FLAGS, "-DEARN_PF_TIMELINE", "-c", os.path.join(earn_build.CSRC, "prefill.hip"),
                        "-o", obj], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for the timeline variant of prefill.hip:\n" + r.stderr)
    objs = [obj if o.endswith(os.sep + "prefill.o") else o for o in objs]
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", TIMELINE_LIB, *objs], check=True)
    return TIMELINE_LIB


def main(argv) -> int:
    name = argv[1] if len(argv) > 1 else "mid_mha"
    from . import binding as B, workloads as W
    cfg = W.CONFIGS[name]
    w = W.Workload(cfg)
    if cfg.dtype != "bf16" or w.max_seqlen <= 64 or not (w.max_seqlen <= 3072 or w.total_tokens // cfg.batch <= 2048):
        print(f"{name}: its full-length layers do not run prefill_mfma_kernel<D,4,2> (the kernel with the timers)")
        return 2
    B.LIB_PATH = build_timeline_library()
    dev = "cuda:0"
    desc = B.make_desc(torch.bfloat16, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, 0.0, cfg.rope_base)
    T = w.total_tokens
    g = torch.Generator(device=dev)
    g.manual_seed(1)
    mk = lambda h: torch.randn(T, h, cfg.head_dim, device=dev, dtype=torch.bfloat16, generator=g)
    q, k, v = mk(cfg.n_q_heads), mk(cfg.n_kv_heads), mk(cfg.n_kv_heads)
    out, kr = torch.empty_like(q), torch.empty_like(k)
    cu = torch.tensor(w.cu_seqlens, dtype=torch.int32, device=dev)
    ws = torch.empty(max(B.earn_prefill_workspace_bytes(desc, cfg.batch, T, w.max_seqlen, True), 256), dtype=torch.uint8,
                     device=dev)
    run = lambda: B.earn_prefill_attn(desc, q, k, v, cu, None, cfg.batch, T, w.max_seqlen, out, kr, None, ws)
    for _ in range(3):
        run()
    torch.cuda.synchronize()
    L = B.lib()
    L.earn_debug_set_timeline.argtypes = [ctypes.c_void_p, ctypes.c_int]
    slots = 1 << 18
    buf = torch.zeros(slots * 8, dtype=torch.int64, device=dev)
    assert L.earn_debug_set_timeline(buf.data_ptr(), slots) == 0
    run()
    torch.cuda.synchronize()
    assert L.earn_debug_set_timeline(None, 0) == 0
    a = buf.cpu().numpy().reshape(slots, 8)
    a = a[a[:, 0] > 0]
    val, emp = a[a[:, 7] > 0], a[a[:, 7] == 0]
    t0 = a[:, 0].min()
    span = (max(val[:, 5].max(), a[:, 0].max()) - t0) * TICK_US
    d = lambda i, j: (val[:, j] - val[:, i]) * TICK_US
    tiles = val[:, 7]
    print(f"{name}: one full-length layer, prefill_mfma_kernel<{cfg.head_dim},4,2> with timers: {len(a)} workgroups launched, "
          f"{len(val)} with a block inside their sequence, {len(emp)} beyond it; {span:.0f} us from the first entry to the last store")
    print(f"life of a workgroup (mean over those with a block, {tiles.mean():.1f} tiles of 64 keys each): {d(0, 5).mean():.1f} us =")
    print(f"  {d(0, 1).mean():.2f} us  kernel arguments -> sequence bounds -> block known")
    print(f"  {d(1, 2).mean():.2f} us  until the query rows, their cos/sin rows and the first K/V tile have arrived")
    print(f"  {d(2, 3).mean():.2f} us  first tile (exact maxima)")
    more = tiles > 1
    print(f"  {d(3, 4).mean():.2f} us  the other tiles: {d(3, 4)[more].sum() / (tiles[more] - 1).sum():.3f} us per tile")
    print(f"  {d(4, 5).mean():.2f} us  normalise and issue the output stores")
    for lo, hi in ((1, 2), (3, 6), (7, 12), (13, 20), (21, 64)):
        m = (tiles >= lo) & (tiles <= hi)
        if m.any():
            rest = d(3, 4)[m].sum() / max((tiles[m] - 1).sum(), 1)
            print(f"  blocks of {lo:2d}-{hi:2d} tiles: {int(m.sum()):6d} workgroups, life {d(0, 5)[m].mean():5.1f} us, before the first tile "
                  f"{d(0, 2)[m].mean():.2f}, first tile {d(2, 3)[m].mean():.2f}, per further tile {rest:.3f}, stores {d(4, 5)[m].mean():.2f}")
    occ, gaps = np.zeros(3), []
    for cu_id in np.unique(val[:, 6]):
        x = val[val[:, 6] == cu_id]
        events = sorted([(t, 1) for t in x[:, 0]] + [(t, -1) for t in x[:, 5]])
        live, last = 0, t0
        for t, step in events:
            occ[min(live, 2)] += t - last
            last, live = t, live + step
        starts, ends = np.sort(x[:, 0]), np.sort(x[:, 5])
        nxt = np.searchsorted(starts, ends, side="left")
        ok = nxt < len(starts)
        gaps.extend(((starts[nxt[ok]] - ends[ok]) * TICK_US).tolist())
    occ /= occ.sum()
    gaps = np.asarray(gaps)
    print(f"a CU holds 2 / 1 / 0 workgroups with a block {occ[2] * 100:.0f} / {occ[1] * 100:.0f} / {occ[0] * 100:.0f} % of the time "
          f"({len(np.unique(val[:, 6]))} CUs seen)")
    print(f"from the last store of a workgroup to the entry of the next one with a block on the same CU: median "
          f"{np.median(gaps):.2f} us, mean {gaps.mean():.2f} us")
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
