"""A decode step of every layer, one launch per layer (the form a real model needs), recorded into a HIP graph: every
replay must give what the eager launches give, with other work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

from paper_2507_00715_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _draw(w, cfg, g):
    return [[w.decode_tensor(what, l, g, device=DEV) for l in range(cfg.n_layers)] for what in ("q", "k", "v")]


@pytest.mark.parametrize("name", ["small_gqa", "tiny_f32"])
def test_decode_step_graph_replays_equal_eager(name):
    from paper_2507_00715_amd import binding as B
    from paper_2507_00715_amd.pipeline import EarnPath, capture_graph
    B.lib()
    cfg = W.CONFIGS[name]
    w = W.Workload(cfg)
    N, kk, G = cfg.n_layers, cfg.split_k, cfg.decode_steps
    path = EarnPath(n_layers=N, split_k=kk, n_head_reg=cfg.n_head_reg, n_tail_reg=cfg.n_tail_reg, n_q_heads=cfg.n_q_heads,
                    n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim, dtype=cfg.torch_dtype, cu_seqlens=w.cu_seqlens,
                    stream_to_seq=w.stream_to_seq, gen_cap=G, rope_base=cfg.rope_base, device=DEV)
    coords = w.token_coords(DEV)
    q, k, v = ([w.prefill_tensor(what, l, coords=coords) for l in range(N)] for what in ("q", "k", "v"))
    path.prefill(q, k, v, None)
    steps = [_draw(w, cfg, g) for g in range(2)]
    # eager reference: steps 0 and 1, outputs of every layer after each
    eager = []
    for g, (dq, dk, dv) in enumerate(steps):
        path.decode_step(g, dq, dk, dv)
        torch.cuda.synchronize()
        eager.append([o.clone() for o in path.decode_out])
    gen_k_ref = [t.clone() for t in path.gen_k]
    # the same two steps from graphs (one graph per step: the step index is baked into the position kernel's arguments)
    for t in path.gen_k + path.gen_v:
        t.zero_()
    graphs = []
    for g, (dq, dk, dv) in enumerate(steps):
        calls = [path.bind_set_step(g)] + [path.bind_decode_layer(l, dq[l], dk[l], dv[l]) for l in range(N)]
        graphs.append(capture_graph(calls))
    scratch = torch.zeros(1 << 20, device=DEV)
    for rep in range(3):
        for t in path.gen_k + path.gen_v:
            t.zero_()
        for g, graph in enumerate(graphs):
            for o in path.decode_out:
                o.fill_(float("nan"))
            graph.replay()
            scratch.add_(1.0).sum().item()           # the program's own eager work and a synchronisation between replays
            torch.cuda.synchronize()
            for l in range(N):
                assert torch.equal(path.decode_out[l], eager[g][l]), f"replay {rep}, step {g}, layer {l}"
        for l in range(N):
            assert torch.equal(path.gen_k[l], gen_k_ref[l])
