"""A schedule run recorded into a HIP graph and replayed: every replay must reproduce the eager results bit for
bit (the library launches kernels only -- no memset nodes, no allocation, no synchronisation -- and its kernels
are deterministic), with eager work and synchronisations between the replays."""
import numpy as np
import pytest

from paper_1908_05460_amd import binding as B, schedule as sch
from tests.gpu_util import rand_inputs, to_gpu

pytestmark = pytest.mark.gpu

STACK = [  # (C, H, K, stride): fused, multi-shape exact, LDS-gather and 2x2-plane shapes, repeated shapes
    (3, 32, 16, 1), (16, 32, 16, 1), (16, 32, 16, 1), (16, 32, 32, 2), (32, 16, 32, 1), (32, 16, 32, 1),
    (64, 8, 128, 1), (128, 4, 256, 1), (128, 4, 256, 1), (64, 2, 128, 1), (64, 2, 128, 1),
]


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_schedule_run_replays_from_a_graph(dtype):
    import torch
    N = 16
    descs = [B.desc(N, C, H, H, K, stride=st, dtype=B.BF16 if dtype == "bf16" else B.F32) for C, H, K, st in STACK]
    data = [rand_inputs(d, 40 + i, dtype) for i, d in enumerate(descs)]
    Xs = [to_gpu(x) for x, _ in data]
    dYs = [to_gpu(y) for _, y in data]
    dWs = [torch.zeros((d.K, d.C, 3, 3), device="cuda") for d in descs]
    s = B.Schedule(descs, Xs, dYs, dWs)
    rng = np.random.default_rng(5)
    masks = [np.full(len(descs), sch.EXACT, np.uint8), np.full(len(descs), sch.APPROX, np.uint8),
             rng.integers(0, 4, len(descs)).astype(np.uint8)]
    ws = B.alloc_workspace(max(s.workspace_bytes(m) for m in masks))
    for m in masks:
        kw = dict(scale=1 / 128, sigma=1 / 128, seed=9, offset=1000)
        s.run(m, ws, **kw)
        torch.cuda.synchronize()
        eager = [t.clone() for t in dWs]
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            s.run(m, ws, **kw)
        for replay in range(3):
            for t in dWs:
                t.fill_(float("nan"))                    # eager work between the replays
            ws.fill_(replay + 1)                         # stale workspace contents must not matter
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for i, (a, b) in enumerate(zip(eager, dWs)):
                assert torch.equal(a, b), (replay, i, STACK[i], int(m[i]))


def test_topk_schedule_replays_from_a_graph():
    import torch
    N = 8
    descs = [B.desc(N, C, H, H, K, stride=st) for C, H, K, st in STACK]
    data = [rand_inputs(d, 90 + i) for i, d in enumerate(descs)]
    dWs = [torch.zeros((d.K, d.C, 3, 3), device="cuda") for d in descs]
    s = B.Schedule(descs, [to_gpu(x) for x, _ in data], [to_gpu(y) for _, y in data], dWs)
    m = np.array([sch.APPROX, sch.EXACT] * 5 + [sch.APPROX], np.uint8)
    ws = B.alloc_workspace(s.workspace_bytes_topk(m, 4))
    s.run_topk(m, 4, ws, scale=0.25)
    torch.cuda.synchronize()
    eager = [t.clone() for t in dWs]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        s.run_topk(m, 4, ws, scale=0.25)
    for replay in range(3):
        for t in dWs:
            t.fill_(float("nan"))
        ws.fill_(replay + 7)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(zip(eager, dWs)):
            assert torch.equal(a, b), (replay, i, STACK[i], int(m[i]))
