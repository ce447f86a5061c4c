"""GPU parity of the producer-side fusion X = RMSNorm(H) * gamma, S = compress(X, v)."""
import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_helpers import (TOL_BF16_STORE, TOL_F32, assert_bf16_store_matches, rel_fro, rel_max, to_dev, to_host_bits,
                         to_host_f64)

pytestmark = pytest.mark.gpu
EPS = float(np.float32(1e-5))


@pytest.fixture(scope="module")
def vl():
    import __graft_entry__ as ge
    ge.ensure_built()
    import paper_2405_17991_amd as vl
    return vl


def _inputs(N, D, dtype, seed):
    H = wl.random_tensor(N, D, dtype, seed, 31, 1.7)
    H[:, :: max(1, D // 7)] = wl.to_storage(np.full((N, len(range(0, D, max(1, D // 7)))), 9.0, np.float32), dtype)  # outlier channels
    gamma = (1.0 + 0.25 * wl.random_tensor(1, D, wl.F32, seed, 32, 1.0)[0]).astype(np.float32)
    return H, gamma


# fused kernel: d/8 (bf16) or d/4 (f32) a power of two <= 64; the rest take the two-launch path
CASES = [(256, 64, 16), (197, 768, 64), (130, 4096, 256), (33, 5120, 256), (65, 4096, 128), (9, 8192, 512),
         (50, 60, 12), (7, 2048, 1024), (3, 16384, 256), (1, 8, 8), (300, 24, 24)]


@pytest.mark.parametrize("N,D,d", CASES)
@pytest.mark.parametrize("dtype", [wl.BF16, wl.F32])
def test_against_oracle(vl, N, D, d, dtype):
    import torch
    M = D // d
    H, gamma = _inputs(N, D, dtype, 2000 + N + D)
    v = wl.random_unit_v(d, 3)
    X_exact, X_store, _, _ = oracle.rmsnorm_compress(H, gamma, EPS, v, M)
    Xd, Sd = vl.velora_rmsnorm_compress(to_dev(H, dtype), to_dev(gamma, wl.F32), EPS, to_dev(v, wl.F32), M)
    torch.cuda.synchronize()
    if dtype == wl.BF16:
        assert rel_fro(to_host_f64(Xd), X_exact) <= TOL_BF16_STORE
        assert_bf16_store_matches(to_host_bits(Xd), X_exact, X_store, "X")
    else:
        assert rel_fro(to_host_f64(Xd), X_exact) <= TOL_F32 and rel_max(to_host_f64(Xd), X_exact) <= TOL_F32
    Xg = to_host_bits(Xd)
    S2_exact, S2_store = oracle.compress(Xg, v, M)
    got = to_host_f64(Sd)
    if dtype == wl.BF16:
        assert rel_fro(got, S2_exact) <= TOL_BF16_STORE
        assert_bf16_store_matches(to_host_bits(Sd), S2_exact, S2_store, "S")
    else:
        assert rel_fro(got, S2_exact) <= TOL_F32 and rel_max(got, S2_exact) <= TOL_F32


@pytest.mark.parametrize("N,D,d", [(256, 4096, 256), (197, 768, 64), (33, 5120, 128), (64, 1024, 8)])
def test_same_bits_as_compress_on_the_stored_activation(vl, N, D, d):
    import torch
    M = D // d
    H, gamma = _inputs(N, D, wl.BF16, 7)
    v = to_dev(wl.random_unit_v(d, 4), wl.F32)
    Xd, Sd = vl.velora_rmsnorm_compress(to_dev(H, wl.BF16), to_dev(gamma, wl.F32), EPS, v, M)
    S2 = vl.velora_compress(Xd, v, M)
    torch.cuda.synchronize()
    assert torch.equal(Sd.view(torch.int16), S2.view(torch.int16))


def test_in_place_over_the_input(vl):
    import torch
    N, D, d = 128, 4096, 256
    H, gamma = _inputs(N, D, wl.BF16, 9)
    v = to_dev(wl.random_unit_v(d, 4), wl.F32)
    gd = to_dev(gamma, wl.F32)
    Xd, Sd = vl.velora_rmsnorm_compress(to_dev(H, wl.BF16), gd, EPS, v, D // d)
    h2 = to_dev(H, wl.BF16)
    X2, S2 = vl.velora_rmsnorm_compress(h2, gd, EPS, v, D // d, X=h2)
    torch.cuda.synchronize()
    assert torch.equal(X2.view(torch.int16), Xd.view(torch.int16)) and torch.equal(S2.view(torch.int16), Sd.view(torch.int16))


def test_full_size_llama7b_attention_input(vl):
    import torch
    sh = wl.shape_by_name("cfg4_attn")
    H, gamma = _inputs(sh.N, sh.D, wl.BF16, 11)
    v = wl.random_unit_v(sh.d, 5)
    Xd, Sd = vl.velora_rmsnorm_compress(to_dev(H, wl.BF16), to_dev(gamma, wl.F32), EPS, to_dev(v, wl.F32), sh.M)
    torch.cuda.synchronize()
    X_exact, X_store, _, _ = oracle.rmsnorm_compress(H, gamma, EPS, v, sh.M)
    Xg = to_host_bits(Xd)
    assert_bf16_store_matches(Xg, X_exact, X_store, "X")
    S2_exact, S2_store = oracle.compress(Xg, v, sh.M)
    assert_bf16_store_matches(to_host_bits(Sd), S2_exact, S2_store, "S")
