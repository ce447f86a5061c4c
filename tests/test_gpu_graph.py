"""The steady-state hot path (compress -> weight_grad) allocates nothing,
synchronises nothing and clears no memory, so it can be captured in a HIP graph.
Every replay is checked against the eager result, with eager work and
synchronisations between the replays."""
import numpy as np
import pytest

import workloads as wl
from gpu_helpers import to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vl():
    import __graft_entry__ as ge
    ge.ensure_built()
    import paper_2405_17991_amd as vl
    return vl


@pytest.mark.parametrize("N,O,D,d", [(4 * 197, 512, 768, 64), (1024, 256, 1376, 32)])
def test_hot_path_replays_from_a_graph(vl, N, O, D, d):
    import torch
    M = D // d
    X = [to_dev(wl.random_tensor(N, D, wl.BF16, seed=s), wl.BF16) for s in (1, 2, 3)]
    G = [to_dev(wl.random_tensor(N, O, wl.BF16, seed=10 + s, sigma=0.02), wl.BF16) for s in (1, 2, 3)]
    v = to_dev(wl.random_unit_v(d, seed=4), wl.F32)
    need = vl.velora_workspace_bytes(vl.OP_WEIGHT_GRAD, N, D, O, M, vl.BF16)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    Xs, Gs = X[0].clone(), G[0].clone()                    # static graph inputs
    S = torch.empty((N, M), dtype=torch.bfloat16, device="cuda")
    dW = torch.empty((O, D), dtype=torch.float32, device="cuda")

    def step():
        vl.velora_compress(Xs, v, M, S=S)
        vl.velora_weight_grad(Gs, S, v, D, dW=dW, ws=ws)

    # eager references for the three input sets
    refs = []
    for x, g in zip(X, G):
        Xs.copy_(x); Gs.copy_(g)
        step()
        torch.cuda.synchronize()
        refs.append((S.clone(), dW.clone()))

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                             # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()

    for rep in range(6):
        i = rep % 3
        Xs.copy_(X[i]); Gs.copy_(G[i])
        dW.fill_(float("nan")); S.fill_(float("nan"))      # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(S, refs[i][0]), f"replay {rep}: S differs from the eager result"
        assert torch.equal(dW, refs[i][1]), f"replay {rep}: dW differs from the eager result"
