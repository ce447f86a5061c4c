"""GPU parity of the producer-side fusion X = silu(gate) * up, S = compress(X, v)."""
import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_helpers import (TOL_BF16_STORE, TOL_F32, assert_bf16_store_matches, rel_fro, rel_max, to_dev, to_host_bits,
                         to_host_f64)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vl():
    import __graft_entry__ as ge
    ge.ensure_built()
    import paper_2405_17991_amd as vl
    return vl


def _inputs(N, D, dtype, seed):
    gate = wl.random_tensor(N, D, dtype, seed, 21, 2.0)      # pre-activations a few units wide: both silu branches
    up = wl.random_tensor(N, D, dtype, seed, 22, 1.0)
    return gate, up


CASES = [(256, 64, 16), (197, 768, 64), (130, 1376, 32), (33, 4096, 1024), (7, 2048, 2048), (64, 96, 8), (50, 60, 12),
         (1, 8, 8), (300, 24, 24), (97, 2 * 344, 344), (45, 2 * 1032, 1032), (131, 120, 40)]


@pytest.mark.parametrize("N,D,d", CASES)
@pytest.mark.parametrize("dtype", [wl.BF16, wl.F32])
def test_against_oracle(vl, N, D, d, dtype):
    import torch
    M = D // d
    gate, up = _inputs(N, D, dtype, 1000 + N + D)
    v = wl.random_unit_v(d, 3)
    X_exact, X_store, S_exact, S_store = oracle.swiglu_compress(gate, up, v, M)
    Xd, Sd = vl.velora_swiglu_compress(to_dev(gate, dtype), to_dev(up, dtype), to_dev(v, wl.F32), M)
    torch.cuda.synchronize()
    if dtype == wl.BF16:
        assert rel_fro(to_host_f64(Xd), X_exact) <= TOL_BF16_STORE
        assert_bf16_store_matches(to_host_bits(Xd), X_exact, X_store, "X")
    else:
        assert rel_fro(to_host_f64(Xd), X_exact) <= TOL_F32 and rel_max(to_host_f64(Xd), X_exact) <= TOL_F32
    # S belongs to the X the GPU actually stored: the oracle's compress on exactly those bits
    Xg = to_host_bits(Xd)
    S2_exact, S2_store = oracle.compress(Xg, v, M)
    got = to_host_f64(Sd)
    if dtype == wl.BF16:
        assert rel_fro(got, S2_exact) <= TOL_BF16_STORE
        assert_bf16_store_matches(to_host_bits(Sd), S2_exact, S2_store, "S")
    else:
        assert rel_fro(got, S2_exact) <= TOL_F32 and rel_max(got, S2_exact) <= TOL_F32


@pytest.mark.parametrize("N,D,d", [(256, 1024, 256), (197, 768, 64), (33, 4096, 1024), (50, 60, 12), (97, 688, 344),
                                    (45, 2064, 1032), (131, 120, 40)])
def test_same_bits_as_compress_on_the_stored_activation(vl, N, D, d):
    import torch
    M = D // d
    gate, up = _inputs(N, D, wl.BF16, 7)
    v = to_dev(wl.random_unit_v(d, 4), wl.F32)
    Xd, Sd = vl.velora_swiglu_compress(to_dev(gate, wl.BF16), to_dev(up, wl.BF16), v, M)
    S2 = vl.velora_compress(Xd, v, M)
    torch.cuda.synchronize()
    assert torch.equal(Sd.view(torch.int16), S2.view(torch.int16))


def test_in_place_over_gate(vl):
    import torch
    N, D, d = 128, 512, 128
    gate, up = _inputs(N, D, wl.BF16, 9)
    v = to_dev(wl.random_unit_v(d, 4), wl.F32)
    g1, u1 = to_dev(gate, wl.BF16), to_dev(up, wl.BF16)
    Xd, Sd = vl.velora_swiglu_compress(g1, u1, v, D // d)
    g2 = to_dev(gate, wl.BF16)
    X2, S2 = vl.velora_swiglu_compress(g2, u1, v, D // d, X=g2)
    torch.cuda.synchronize()
    assert torch.equal(X2.view(torch.int16), Xd.view(torch.int16)) and torch.equal(S2.view(torch.int16), Sd.view(torch.int16))


def test_full_size_llama7b_down_projection(vl):
    import torch
    sh = wl.shape_by_name("cfg4_down")
    gate, up = _inputs(sh.N, sh.D, wl.BF16, 11)
    v = wl.random_unit_v(sh.d, 5)
    Xd, Sd = vl.velora_swiglu_compress(to_dev(gate, wl.BF16), to_dev(up, wl.BF16), to_dev(v, wl.F32), sh.M)
    torch.cuda.synchronize()
    X_exact, X_store, _, _ = oracle.swiglu_compress(gate, up, v, sh.M)
    assert rel_fro(to_host_f64(Xd), X_exact) <= TOL_BF16_STORE
    Xg = to_host_bits(Xd)
    assert_bf16_store_matches(Xg, X_exact, X_store, "X")
    S2_exact, S2_store = oracle.compress(Xg, v, sh.M)
    assert_bf16_store_matches(to_host_bits(Sd), S2_exact, S2_store, "S")
