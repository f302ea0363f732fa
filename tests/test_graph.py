"""Every entry point enqueues plain kernel launches on the caller's stream (no allocation, no memset, no
synchronisation), so a caller may capture them in a HIP graph.  Captured once, replayed several times with
eager work and synchronisations in between; every replay must reproduce the eager result bit for bit."""
import math

import numpy as np
import pytest

from paper_2410_16663_amd import binding as fa
from paper_2410_16663_amd import inputs as I

pytestmark = pytest.mark.gpu


def test_entry_points_replay_from_a_graph():
    import torch
    print("case graph capture and replay", flush=True)
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(901)
    B, H, Nq, Nk, D, N = 2, 4, 600, 900, 128, 256
    dtype = I.BF16
    mk = lambda shape, m=1.0: torch.from_numpy(
        I.f32_to_bits(rng.standard_normal(shape, dtype=np.float32) * np.float32(m), dtype).view(np.int16)).to(dev)
    q, k, v = mk((B, H, Nq, D)), mk((B, H, Nk, D)), mk((B, H, Nk, D))
    q1 = mk((B, H, 1, D))
    w = mk((H * D, N), 1.0 / math.sqrt(H * D))
    scale = 1.0 / math.sqrt(D)
    plan = fa.fa_fwd_splitkv_plan(B, H, 1, Nk, D, 1, dtype, 5)
    ws = torch.empty((plan.workspace_bytes + 3) // 4, dtype=torch.float32, device=dev)
    ws2 = torch.empty_like(ws)
    klen = torch.tensor([700, 333], dtype=torch.int32, device=dev)

    def outputs():
        return dict(o=torch.zeros((B, H, Nq, D), dtype=torch.int16, device=dev),
                    lse=torch.zeros((B, H, Nq), dtype=torch.float32, device=dev),
                    o1=torch.zeros((B, H, 1, D), dtype=torch.int16, device=dev),
                    lse1=torch.zeros((B, H, 1), dtype=torch.float32, device=dev),
                    om=torch.zeros((B, H, Nq, D), dtype=torch.int16, device=dev),
                    lsem=torch.zeros((B, H, Nq), dtype=torch.float32, device=dev),
                    ol=torch.zeros((B, H, Nq, D), dtype=torch.int16, device=dev),
                    lsel=torch.zeros((B, H, Nq), dtype=torch.float32, device=dev),
                    od=torch.zeros((B, H, 1, D), dtype=torch.int16, device=dev),
                    lsed=torch.zeros((B, H, 1), dtype=torch.float32, device=dev),
                    y=torch.zeros((B, Nq, N), dtype=torch.float32, device=dev))

    def enqueue(t, stream):
        fa.fa_fwd(q, k, v, t["o"], t["lse"], B, H, Nq, Nk, D, scale, 1, dtype, stream)
        fa.fa_fwd_splitkv(q1, k, v, t["o1"], t["lse1"], B, H, 1, Nk, D, scale, 1, dtype, 5, ws, plan.workspace_bytes,
                          stream)
        fa.fa_fwd_masked(q, k, v, t["om"], t["lsem"], B, H, Nq, Nk, D, scale, 200, 0, 64, klen, dtype, stream)
        fa.fa_attn_linear(q, k, v, w, t["ol"], t["lsel"], t["y"], B, H, Nq, Nk, D, N, scale, 1, dtype, 256, stream)
        fa.fa_decode_masked(q1, k, v, t["od"], t["lsed"], B, H, Nk, D, scale, 300, 0, 32, klen, dtype, 5, ws2,
                            plan.workspace_bytes, stream)

    eager = outputs()
    enqueue(eager, torch.cuda.current_stream().cuda_stream)        # also loads the kernels before any capture
    torch.cuda.synchronize()

    captured = outputs()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            enqueue(captured, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    for replay in range(3):
        for t in captured.values():
            t.zero_()                                              # eager work between replays
        ws.fill_(float("nan"))
        ws2.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, t in captured.items():
            assert torch.equal(t, eager[name]), (replay, name)
