"""Seeded random shapes through every entry point: a net for tile-selection and
edge-handling mistakes that the hand-picked cases might miss.  Shapes are small
enough for the brute-force oracle."""
import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_helpers import (TOL_BF16_STORE, TOL_F32, TOL_F32_FROM_BF16, assert_bf16_store_matches, rel_fro, rel_max,
                         to_dev, to_host_bits, to_host_f64)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vl():
    import __graft_entry__ as ge
    ge.ensure_built()
    import paper_2405_17991_amd as vl
    return vl


def _shapes(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    d_choices = [1, 2, 3, 4, 5, 8, 12, 16, 24, 32, 64, 100, 128, 256, 512, 1024]
    for _ in range(n):
        d = int(rng.choice(d_choices))
        M = int(rng.integers(1, max(2, min(300, 6000 // d))))
        N = int(rng.integers(1, 700))
        O = int(rng.integers(1, 40)) * int(rng.choice([1, 2, 4, 8]))
        dtype = wl.BF16 if rng.random() < 0.7 else wl.F32
        out.append((N, O, M * d, d, dtype))
    return out


@pytest.mark.parametrize("N,O,D,d,dtype", _shapes(40, 2024))
def test_random_shape(vl, N, O, D, d, dtype):
    M = D // d
    seed = N * 7919 + O * 104729 + D
    X = wl.random_tensor(N, D, dtype, seed=seed, stream=6)
    G = wl.random_tensor(N, O, dtype, seed=seed, stream=7, sigma=0.05)
    v = wl.random_unit_v(d, seed=seed)
    Xd, Gd, vd = to_dev(X, dtype), to_dev(G, dtype), to_dev(v, wl.F32)
    # compress
    S = vl.velora_compress(Xd, vd, M)
    S_exact, S_store = oracle.compress(X, v, M)
    if dtype == wl.F32:
        assert rel_fro(to_host_f64(S), S_exact) <= TOL_F32 and rel_max(to_host_f64(S), S_exact) <= TOL_F32
    else:
        assert rel_fro(to_host_f64(S), S_exact) <= TOL_BF16_STORE
        assert_bf16_store_matches(to_host_bits(S), S_exact, S_store, "compress")
    # weight gradient from the oracle's stored S
    dW = vl.velora_weight_grad(Gd, to_dev(S_store, dtype), vd, D)
    want = oracle.weight_grad_bruteforce(G, S_store, v, D)
    tol = TOL_F32 if dtype == wl.F32 else TOL_F32_FROM_BF16
    assert rel_fro(to_host_f64(dW), want) <= tol and rel_max(to_host_f64(dW), want) <= tol
    # reconstruct
    Xhat = vl.velora_reconstruct(to_dev(S_store, dtype), vd, D)
    ref = oracle.reconstruct(S_store, v, D)
    if dtype == wl.F32:
        assert np.abs(to_host_f64(Xhat) - ref).max() <= 2.0 ** -23 * max(np.abs(ref).max(), 1e-30)
    else:
        assert (np.abs(to_host_f64(Xhat) - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-30).all()


def _wide_output_shapes(n, seed):
    # more than 8192 output features: the weight gradient's 256-feature tiles for up to 80 sub-tokens per
    # token, the 128-feature kernels on the same plan beyond that or when O is not a multiple of 8
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        d = int(rng.choice([8, 16, 32, 64]))
        M = int(rng.integers(1, min(100, 2048 // d) + 1))
        N = int(rng.integers(1, 1000))
        O = 8192 + int(rng.integers(1, 160)) * int(rng.choice([8, 8, 8, 4, 1]))
        out.append((N, O, M * d, d))
    return out


@pytest.mark.parametrize("N,O,D,d", _wide_output_shapes(16, 77))
def test_random_shape_wide_output_weight_grad(vl, N, O, D, d):
    M = D // d
    seed = N * 7919 + O * 104729 + D
    G = wl.random_tensor(N, O, wl.BF16, seed=seed, stream=7, sigma=0.05)
    S = wl.random_tensor(N, M, wl.BF16, seed=seed, stream=8)
    v = wl.random_unit_v(d, seed=seed)
    dW = vl.velora_weight_grad(to_dev(G, wl.BF16), to_dev(S, wl.BF16), to_dev(v, wl.F32), D)
    want = oracle.weight_grad_bruteforce(G, S, v, D)
    got = to_host_f64(dW)
    assert rel_fro(got, want) <= TOL_F32_FROM_BF16 and rel_max(got, want) <= TOL_F32_FROM_BF16


def _gemm_shapes(n, seed):
    # multiples that reach the MFMA kernel (D % 64 == 0 and O % 4 == 0 forward, O % 64 == 0 and D % 8 == 0
    # backward) mixed with ones that do not
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        d = int(rng.choice([8, 16, 32, 64, 64, 128, 192, 256]))
        M = int(rng.integers(1, max(2, 1100 // d)))
        D = M * d
        N = int(rng.integers(1, 900))
        O = int(rng.integers(1, 12)) * int(rng.choice([1, 4, 8, 64, 64]))
        dtype = wl.BF16 if rng.random() < 0.8 else wl.F32
        out.append((N, O, D, d, dtype))
    return out


@pytest.mark.parametrize("N,O,D,d,dtype", _gemm_shapes(30, 77))
def test_random_shape_dense_products(vl, N, O, D, d, dtype):
    """velora_linear_compress and velora_grad_input on seeded random shapes."""
    import torch
    M = D // d
    seed = N * 7919 + O * 104729 + D
    X = wl.random_tensor(N, D, dtype, seed=seed, stream=6)
    W = wl.random_tensor(O, D, dtype, seed=seed, stream=8, sigma=D ** -0.5)
    G = wl.random_tensor(N, O, dtype, seed=seed, stream=7, sigma=0.05)
    v = wl.random_unit_v(d, seed=seed)
    Yd, Sd = vl.velora_linear_compress(to_dev(X, dtype), to_dev(W, dtype), to_dev(v, wl.F32), M)
    dXd = vl.velora_grad_input(to_dev(G, dtype), to_dev(W, dtype))
    torch.cuda.synchronize()
    Y_exact, Y_store, S_exact, S_store = oracle.linear_compress(X, W, v, M)
    dX_exact, dX_store = oracle.grad_input(G, W)
    if dtype == wl.F32:
        for got, want in ((Yd, Y_exact), (Sd, S_exact), (dXd, dX_exact)):
            assert rel_fro(to_host_f64(got), want) <= TOL_F32 and rel_max(to_host_f64(got), want) <= TOL_F32
    else:
        assert_bf16_store_matches(to_host_bits(Yd), Y_exact, Y_store, "Y")
        assert_bf16_store_matches(to_host_bits(Sd), S_exact, S_store, "S")
        assert_bf16_store_matches(to_host_bits(dXd), dX_exact, dX_store, "dX")
