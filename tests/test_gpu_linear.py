"""The layer's forward with the compression taken from the same pass
(velora_linear_compress: paper Listing 1, forward, and Sec. 3.1) against the
CPU oracle: Y = X @ W^T and S = compress(X, v), element by element."""
import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_helpers import (TOL_BF16, TOL_BF16_STORE, TOL_F32, assert_bf16_store_matches, rel_fro, rel_max, to_dev,
                         to_host_bits, to_host_f64)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vl():
    import __graft_entry__ as ge
    ge.ensure_built()
    import paper_2405_17991_amd as vl
    return vl


def _rows_in_every_token_tile(N, seed, tile=256):
    """One seeded token row inside every tile of `tile` tokens (the GEMM's block height), plus the first
    and last rows of the array and both sides of the first tile edge: a tile the block-id mapping skipped
    or wrote twice cannot hide between samples."""
    rng = np.random.default_rng(seed)
    rows = {0, 1, min(N - 1, tile - 1), min(N - 1, tile), N - 2 if N > 1 else 0, N - 1}
    for t0 in range(0, N, tile):
        rows.add(int(t0 + rng.integers(0, min(tile, N - t0))))
    return np.array(sorted(rows))


def _inputs(N, D, O, d, dtype, seed):
    X = wl.random_tensor(N, D, dtype, seed, 31, 1.0)
    W = wl.random_tensor(O, D, dtype, seed, 32, D ** -0.5)
    v = wl.random_unit_v(d, seed + 1)
    return X, W, v


def _check(vl, N, D, O, d, dtype, seed=0):
    import torch
    M = D // d
    X, W, v = _inputs(N, D, O, d, dtype, 500 + seed + N + D + O)
    Y_exact, Y_store, S_exact, S_store = oracle.linear_compress(X, W, v, M)
    Yd, Sd = vl.velora_linear_compress(to_dev(X, dtype), to_dev(W, dtype), to_dev(v, wl.F32), M)
    torch.cuda.synchronize()
    assert tuple(Yd.shape) == (N, O) and tuple(Sd.shape) == (N, M)
    Y, S = to_host_f64(Yd), to_host_f64(Sd)
    if dtype == wl.F32:
        assert rel_fro(Y, Y_exact) <= TOL_F32 and rel_max(Y, Y_exact) <= TOL_F32
        assert rel_fro(S, S_exact) <= TOL_F32 and rel_max(S, S_exact) <= TOL_F32
    else:
        assert rel_fro(Y, Y_exact) <= TOL_BF16 and rel_fro(Y, Y_exact) <= TOL_BF16_STORE
        assert rel_fro(S, S_exact) <= TOL_BF16 and rel_fro(S, S_exact) <= TOL_BF16_STORE
        assert_bf16_store_matches(to_host_bits(Yd), Y_exact, Y_store, "Y")
        assert_bf16_store_matches(to_host_bits(Sd), S_exact, S_store, "S")
    return Yd, Sd


# bf16, D % 64 == 0, O % 4 == 0, d % 64 == 0: the MFMA kernel forms S itself.  Ragged token and output
# tiles, one and several k steps, one and several sub-tokens per k step range, the largest fused d.
FUSED = [(300, 128, 260, 64), (512, 256, 512, 128), (256, 64, 256, 64), (700, 192, 100, 64), (131, 2048, 64, 2048),
         (130, 4096, 68, 1024), (1, 64, 4, 64), (1030, 320, 1028, 64), (2304, 128, 2048, 128),
         # sub-tokens shared out over the output tiles: more sub-tokens than tiles (7 over 3), several k steps each
         (300, 448, 600, 64), (260, 768, 520, 128), (257, 1536, 1024, 256), (300, 4096, 520, 2048)]
# bf16 MFMA kernel for Y, compress kernel for S (d not a multiple of 64)
UNFUSED = [(300, 128, 260, 32), (200, 704, 36, 88), (64, 4096, 8, 4096), (90, 64, 256, 8)]
# everything else: plain FMA kernel (D % 64 != 0, O % 4 != 0)
GENERIC = [(100, 96, 50, 32), (64, 128, 37, 64), (33, 60, 9, 12), (5, 8, 3, 8)]


@pytest.mark.parametrize("N,D,O,d", FUSED + UNFUSED + GENERIC)
def test_bf16_against_oracle(vl, N, D, O, d):
    _check(vl, N, D, O, d, wl.BF16)


@pytest.mark.parametrize("N,D,O,d", [(256, 64, 64, 16), (77, 63, 19, 7), (130, 128, 70, 64), (1, 1, 1, 1)])
def test_f32_against_oracle(vl, N, D, O, d):
    _check(vl, N, D, O, d, wl.F32)


@pytest.mark.parametrize("N,D,O,d", [(300, 128, 260, 64), (512, 512, 256, 256)])
def test_s_agrees_with_the_compress_kernel(vl, N, D, O, d):
    # inside the GEMM v enters as the sum of two bf16 numbers: S may differ from velora_compress in the last
    # bf16 digit where the dot is within ~1e-5 of a rounding boundary, nowhere by more
    import torch
    from gpu_helpers import bf16_ordered
    X, W, v = _inputs(N, D, O, d, wl.BF16, 77)
    Xd, vd = to_dev(X, wl.BF16), to_dev(v, wl.F32)
    _, S1 = vl.velora_linear_compress(Xd, to_dev(W, wl.BF16), vd, D // d)
    S2 = vl.velora_compress(Xd, vd, D // d)
    torch.cuda.synchronize()
    dist = np.abs(bf16_ordered(to_host_bits(S1)) - bf16_ordered(to_host_bits(S2)))
    exact = to_host_f64(S2)
    big = np.abs(exact) >= 1e-3 * np.sqrt(np.mean(exact * exact))
    assert dist[big].max() <= 1 and (dist[big] != 0).mean() <= 2e-2


def test_unaligned_pointers_take_the_generic_path(vl):
    import torch
    N, D, O, d = 70, 128, 64, 64
    X, W, v = _inputs(N, D, O, d, wl.BF16, 5)
    buf = torch.empty(N * D + 1, dtype=torch.bfloat16, device="cuda")
    Xd = buf[1:].view(N, D)                      # 2-byte aligned only
    Xd.copy_(to_dev(X, wl.BF16))
    Yd, Sd = vl.velora_linear_compress(Xd, to_dev(W, wl.BF16), to_dev(v, wl.F32), D // d)
    torch.cuda.synchronize()
    Y_exact, Y_store, S_exact, S_store = oracle.linear_compress(X, W, v, D // d)
    assert_bf16_store_matches(to_host_bits(Yd), Y_exact, Y_store, "Y")
    assert_bf16_store_matches(to_host_bits(Sd), S_exact, S_store, "S")


def test_identity_weight_copies_the_input(vl):
    # W = I: Y = X bit for bit (one non-zero product per output, exact in float32)
    import torch
    N, D = 300, 128
    X = wl.random_tensor(N, D, wl.BF16, 9)
    W = wl.to_storage(np.eye(D, dtype=np.float32), wl.BF16)
    v = wl.random_unit_v(64, 2)
    Yd, _ = vl.velora_linear_compress(to_dev(X, wl.BF16), to_dev(W, wl.BF16), to_dev(v, wl.F32), 2)
    torch.cuda.synchronize()
    assert np.array_equal(to_host_bits(Yd), X)


def test_full_size_sampled(vl):
    # the LLaMA-7B-like down projection at its real size; the oracle computes one token row of every 256-token tile
    import torch
    sh = wl.shape_by_name("cfg4_down")
    torch.manual_seed(0)
    Xd = (torch.randn((sh.N, sh.D), device="cuda") * 1.0).to(torch.bfloat16)
    Wd = (torch.randn((sh.O, sh.D), device="cuda") * sh.D ** -0.5).to(torch.bfloat16)
    v = wl.random_unit_v(sh.d, 3)
    Yd, Sd = vl.velora_linear_compress(Xd, Wd, to_dev(v, wl.F32), sh.M)
    torch.cuda.synchronize()
    rows = _rows_in_every_token_tile(sh.N, 11)
    Xs = to_host_bits(Xd[torch.from_numpy(rows).cuda()])
    W = to_host_bits(Wd)
    Y_exact, Y_store, S_exact, S_store = oracle.linear_compress(Xs, W, v, sh.M)
    idx = torch.from_numpy(rows).cuda()
    assert_bf16_store_matches(to_host_bits(Yd[idx]), Y_exact, Y_store, "Y rows")
    assert_bf16_store_matches(to_host_bits(Sd[idx]), S_exact, S_store, "S rows")
    # every S against the stand-alone kernel (property at full size)
    S2 = vl.velora_compress(Xd, to_dev(v, wl.F32), sh.M)
    torch.cuda.synchronize()
    assert rel_fro(to_host_f64(Sd), to_host_f64(S2)) <= 2e-3


# ------------------------------------------------------------------ grad_input = grad_output @ weight
def _check_grad_input(vl, N, O, D, dtype, seed=0):
    import torch
    G = wl.random_tensor(N, O, dtype, 900 + seed + N + O, 41, 0.05)
    W = wl.random_tensor(O, D, dtype, 901 + seed + D, 42, O ** -0.5)
    dX_exact, dX_store = oracle.grad_input(G, W)
    dXd = vl.velora_grad_input(to_dev(G, dtype), to_dev(W, dtype))
    torch.cuda.synchronize()
    assert tuple(dXd.shape) == (N, D)
    got = to_host_f64(dXd)
    if dtype == wl.F32:
        assert rel_fro(got, dX_exact) <= TOL_F32 and rel_max(got, dX_exact) <= TOL_F32
    else:
        assert rel_fro(got, dX_exact) <= TOL_BF16 and rel_fro(got, dX_exact) <= TOL_BF16_STORE
        assert_bf16_store_matches(to_host_bits(dXd), dX_exact, dX_store, "dX")


# MFMA kernel: O % 64 == 0 (the reduction), D % 8 == 0; ragged token and column tiles, one and several k steps
@pytest.mark.parametrize("N,O,D", [(300, 128, 264), (512, 256, 512), (256, 64, 256), (700, 192, 104), (1, 64, 8),
                                   (131, 2048, 72), (1030, 320, 1032), (2304, 128, 2048)])
def test_grad_input_bf16_mfma(vl, N, O, D):
    _check_grad_input(vl, N, O, D, wl.BF16)


@pytest.mark.parametrize("N,O,D", [(100, 96, 50), (64, 37, 128), (33, 9, 60), (5, 3, 8), (70, 128, 36)])
def test_grad_input_bf16_generic(vl, N, O, D):
    _check_grad_input(vl, N, O, D, wl.BF16)


@pytest.mark.parametrize("N,O,D", [(256, 64, 64), (77, 19, 63), (130, 70, 128), (1, 1, 1)])
def test_grad_input_f32(vl, N, O, D):
    _check_grad_input(vl, N, O, D, wl.F32)


def test_grad_input_selects_weight_rows(vl):
    # G = one-hot rows: dX[n, :] = W[o(n), :] bit for bit (pins the [O, D] layout of W and the transposition)
    import torch
    N, O, D = 300, 128, 264
    W = wl.random_tensor(O, D, wl.BF16, 13)
    pick = (np.arange(N) * 7 + 3) % O
    G32 = np.zeros((N, O), dtype=np.float32)
    G32[np.arange(N), pick] = 1.0
    dXd = vl.velora_grad_input(to_dev(wl.to_storage(G32, wl.BF16), wl.BF16), to_dev(W, wl.BF16))
    torch.cuda.synchronize()
    assert np.array_equal(to_host_bits(dXd), W[pick])


def test_grad_input_full_size_sampled(vl):
    import torch
    sh = wl.shape_by_name("cfg4_down")
    torch.manual_seed(1)
    Gd = (torch.randn((sh.N, sh.O), device="cuda") * 0.05).to(torch.bfloat16)
    Wd = (torch.randn((sh.O, sh.D), device="cuda") * sh.O ** -0.5).to(torch.bfloat16)
    dXd = vl.velora_grad_input(Gd, Wd)
    torch.cuda.synchronize()
    rows = _rows_in_every_token_tile(sh.N, 12)
    idx = torch.from_numpy(rows).cuda()
    dX_exact, dX_store = oracle.grad_input(to_host_bits(Gd[idx]), to_host_bits(Wd))
    assert_bf16_store_matches(to_host_bits(dXd[idx]), dX_exact, dX_store, "dX rows")


@pytest.mark.parametrize("name", ["cfg2_vit_fc1", "cfg3_up", "cfg4_up", "cfg5_down_d256", "paper7b_down_m32", "cfg5_up_d64"])
def test_dense_products_at_other_full_sizes_sampled(vl, name):
    """Forward (with S) and input gradient at the real layer sizes of the other configurations; the oracle
    computes one token row of every 256-token tile (plus tile edges, first and last rows)."""
    import torch
    sh = wl.shape_by_name(name)
    torch.manual_seed(sh.N % 97)
    Xd = torch.randn((sh.N, sh.D), device="cuda").to(torch.bfloat16)
    Wd = (torch.randn((sh.O, sh.D), device="cuda") * sh.D ** -0.5).to(torch.bfloat16)
    Gd = (torch.randn((sh.N, sh.O), device="cuda") * 0.05).to(torch.bfloat16)
    v = wl.random_unit_v(sh.d, 3)
    Yd, Sd = vl.velora_linear_compress(Xd, Wd, to_dev(v, wl.F32), sh.M)
    dXd = vl.velora_grad_input(Gd, Wd)
    torch.cuda.synchronize()
    rows = _rows_in_every_token_tile(sh.N, sh.N % 89)
    idx = torch.from_numpy(rows).cuda()
    W = to_host_bits(Wd)
    Y_exact, Y_store, S_exact, S_store = oracle.linear_compress(to_host_bits(Xd[idx]), W, v, sh.M)
    assert_bf16_store_matches(to_host_bits(Yd[idx]), Y_exact, Y_store, "Y rows")
    assert_bf16_store_matches(to_host_bits(Sd[idx]), S_exact, S_store, "S rows")
    dX_exact, dX_store = oracle.grad_input(to_host_bits(Gd[idx]), W)
    assert_bf16_store_matches(to_host_bits(dXd[idx]), dX_exact, dX_store, "dX rows")
