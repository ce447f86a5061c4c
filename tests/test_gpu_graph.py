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


def test_other_entry_points_replay_from_a_graph(vl):
    """The producer-side fusions, the per-batch-v update and the optimiser step are capturable too:
    no allocation, no synchronisation, no memset inside any of them."""
    import torch
    N, D, d, O = 512, 1024, 128, 384
    M = D // d
    gate = [to_dev(wl.random_tensor(N, D, wl.BF16, seed=s, stream=41, sigma=2.0), wl.BF16) for s in (1, 2)]
    up = [to_dev(wl.random_tensor(N, D, wl.BF16, seed=s, stream=42), wl.BF16) for s in (1, 2)]
    gamma = to_dev(np.linspace(0.5, 1.5, D).astype(np.float32), wl.F32)
    v = to_dev(wl.random_unit_v(d, seed=4), wl.F32)
    gs, us_ = gate[0].clone(), up[0].clone()                     # static graph inputs
    X1 = torch.empty((N, D), dtype=torch.bfloat16, device="cuda"); S1 = torch.empty((N, M), dtype=torch.bfloat16, device="cuda")
    X2 = torch.empty_like(X1); S2 = torch.empty_like(S1); S3 = torch.empty_like(S1)
    state0 = torch.full((d,), 0.25, device="cuda")
    state = state0.clone(); v_next = torch.empty(d, device="cuda")
    need = vl.velora_workspace_bytes(vl.OP_INIT_V, N, D, 0, M, vl.BF16)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    T = to_dev(wl.random_tensor(O, M, wl.F32, seed=9, stream=43, sigma=0.02), wl.F32)
    W0 = to_dev(wl.random_tensor(O, D, wl.F32, seed=9, stream=44, sigma=0.05), wl.F32)
    W = W0.clone(); m = torch.zeros_like(W); u = torch.zeros_like(W)

    def reset():
        state.copy_(state0); W.copy_(W0); m.zero_(); u.zero_()

    def step():
        vl.velora_swiglu_compress(gs, us_, v, M, X=X1, S=S1)
        vl.velora_rmsnorm_compress(gs, gamma, 1e-5, v, M, X=X2, S=S2)
        vl.velora_compress_update(X1, v, M, mean_state=state, beta=0.5, S=S3, v_out=v_next, ws=ws)
        vl.velora_adamw_step_factor(T, v_next, W, m, u, lr=1e-2, step=1)

    refs = []
    for g_, u_ in zip(gate, up):
        gs.copy_(g_); us_.copy_(u_); reset()
        step()
        torch.cuda.synchronize()
        refs.append([t.clone() for t in (X1, S1, X2, S2, S3, state, v_next, W, m, u)])

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        reset(); step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    reset()
    with torch.cuda.graph(graph):
        step()
    for rep in range(4):
        i = rep % 2
        gs.copy_(gate[i]); us_.copy_(up[i]); reset()
        for t in (X1, S1, X2, S2, S3):
            t.fill_(float("nan"))                                # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, got, ref in zip(("X1", "S1", "X2", "S2", "S3", "state", "v_next", "W", "m", "u"),
                                  (X1, S1, X2, S2, S3, state, v_next, W, m, u), refs[i]):
            assert torch.equal(got, ref), f"replay {rep}: {name} differs from the eager result"


def test_gemm_entry_points_replay_from_a_graph(vl):
    """velora_linear_compress and velora_grad_input are capturable as well (their one-off per-device set-up
    happens on the warm-up call before the capture)."""
    import torch
    N, D, O, d = 520, 256, 264, 64
    M = D // d
    Xs = [to_dev(wl.random_tensor(N, D, wl.BF16, seed=s, stream=51), wl.BF16) for s in (1, 2)]
    Gs = [to_dev(wl.random_tensor(N, O, wl.BF16, seed=s, stream=52, sigma=0.05), wl.BF16) for s in (1, 2)]
    W = to_dev(wl.random_tensor(O, D, wl.BF16, seed=3, stream=53, sigma=D ** -0.5), wl.BF16)
    v = to_dev(wl.random_unit_v(d, seed=4), wl.F32)
    X, G = Xs[0].clone(), Gs[0].clone()
    Y = torch.empty((N, O), dtype=torch.bfloat16, device="cuda"); S = torch.empty((N, M), dtype=torch.bfloat16, device="cuda")
    dX = torch.empty((N, D), dtype=torch.bfloat16, device="cuda")

    def step():
        vl.velora_linear_compress(X, W, v, M, Y=Y, S=S)
        vl.velora_grad_input(G, W, dX=dX)

    refs = []
    for x_, g_ in zip(Xs, Gs):
        X.copy_(x_); G.copy_(g_)
        step()
        torch.cuda.synchronize()
        refs.append([t.clone() for t in (Y, S, dX)])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(4):
        i = rep % 2
        X.copy_(Xs[i]); G.copy_(Gs[i])
        for t in (Y, S, dX):
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, got, ref in zip(("Y", "S", "dX"), (Y, S, dX), refs[i]):
            assert torch.equal(got, ref), f"replay {rep}: {name} differs from the eager result"
