"""GPU parity: libvelora (through its C ABI) against the CPU oracle, element by
element on the same seeded inputs.  Sizes here are ones the oracle finishes in
seconds but that still span several tiles, ragged tails and every kernel
variant (vectorised / generic, each MFMA tiling, the float32 path)."""
import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_helpers import (TOL_BF16, TOL_BF16_STORE, TOL_F32, TOL_F32_FROM_BF16, assert_bf16_store_matches,
                         rel_fro, rel_max, to_dev, to_host_bits, to_host_f64)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vl():
    import __graft_entry__ as ge
    ge.ensure_built()
    import paper_2405_17991_amd as vl
    return vl


def _torch():
    import torch
    return torch


# ------------------------------------------------------------------ compress
COMPRESS_CASES = [
    # (N, D, d, dtype)  -- d spans every lane grouping of the vectorised kernel
    (256, 64, 16, wl.F32),          # configuration 1
    (37, 64, 4, wl.F32), (129, 96, 8, wl.F32), (300, 128, 32, wl.F32), (77, 192, 64, wl.F32),
    (65, 256, 128, wl.F32), (33, 512, 256, wl.F32), (19, 1024, 512, wl.F32), (9, 2048, 1024, wl.F32),
    (301, 64, 8, wl.BF16), (257, 64, 16, wl.BF16), (130, 96, 32, wl.BF16), (4 * 197, 768, 64, wl.BF16),
    (515, 768, 128, wl.BF16), (203, 1024, 256, wl.BF16), (67, 1536, 512, wl.BF16), (41, 2048, 1024, wl.BF16),
    (23, 4096, 2048, wl.BF16),
    # 16-byte vectors per sub-token not a power of two: the vectorised kernel with idle lanes
    (203, 72, 24, wl.BF16), (131, 120, 40, wl.BF16), (97, 2 * 344, 344, wl.BF16), (515, 3 * 344, 344, wl.F32),
    (67, 2 * 776, 776, wl.BF16), (45, 2 * 1032, 1032, wl.BF16), (29, 2040, 2040, wl.BF16), (33, 3 * 12, 12, wl.F32),
    (21, 2 * 1020, 1020, wl.F32), (150, 11008, 344, wl.BF16),
    # bf16 sub-token sizes that are a multiple of 4 but not of 8: 8-byte vectors
    (97, 2 * 172, 172, wl.BF16), (150, 11008, 172, wl.BF16), (203, 5 * 4, 4, wl.BF16), (131, 3 * 20, 20, wl.BF16),
    (45, 2 * 1028, 1028, wl.BF16), (64, 11008, 1376, wl.BF16), (64, 11008, 688, wl.BF16),
    # ... of 132 to 256 elements are taken in pairs (a pair is d / 4 whole 16-byte vectors): the smallest
    # and the largest such d, a number of pairs that is not a multiple of the eight a wave takes, one pair,
    # and an odd number of sub-tokens (which stays with the 8-byte kernel)
    (5, 10 * 132, 132, wl.BF16), (7, 10 * 252, 252, wl.BF16), (37, 6 * 172, 172, wl.BF16), (1, 2 * 172, 172, wl.BF16),
    (3, 3 * 172, 172, wl.BF16), (9, 2 * 260, 260, wl.BF16),
    # sub-token sizes no vector kernel takes, in an X that is a whole number of 16-byte vectors: tiles of 256 or
    # 64 sub-tokens through LDS (d = 43 and 86 are 256 and 128 sub-tokens per token on the 11008-wide layer,
    # d = 54 and 27 on the 13824-wide one); partial last tiles, fewer sub-tokens than one tile, d = 1, 2, 3,
    # the largest d of each tile size, float32
    (300, 11008, 43, wl.BF16), (150, 11008, 86, wl.BF16), (96, 13824, 54, wl.BF16), (40, 13824, 27, wl.BF16),
    (64, 24, 3, wl.BF16), (1000, 16, 2, wl.BF16), (8, 9, 9, wl.BF16), (16, 127, 127, wl.BF16), (8, 2 * 250, 250, wl.BF16),
    (8, 495, 495, wl.BF16), (8, 497, 497, wl.BF16), (300, 1376 * 2, 43, wl.F32), (52, 300, 100, wl.F32), (4, 3 * 63, 63, wl.F32),
    (4, 250, 250, wl.F32), (2048, 8, 1, wl.BF16),
    # generic kernel: d not a power of two times the vector width, d = 1, d = D
    (50, 60, 12, wl.BF16), (50, 63, 7, wl.F32), (31, 33, 1, wl.BF16), (17, 100, 100, wl.F32),
    (11, 3000, 3000, wl.BF16), (1, 8, 8, wl.BF16), (1, 1, 1, wl.F32),
]


@pytest.mark.parametrize("N,D,d,dtype", COMPRESS_CASES)
def test_compress_matches_oracle(vl, N, D, d, dtype):
    M = D // d
    X = wl.random_tensor(N, D, dtype, seed=N + D + d)
    v = wl.random_unit_v(d, seed=d)
    S = vl.velora_compress(to_dev(X, dtype), to_dev(v, wl.F32), M)
    _torch().cuda.synchronize()
    S_exact, S_store = oracle.compress(X, v, M)
    got = to_host_f64(S)
    if dtype == wl.F32:
        assert rel_fro(got, S_exact) <= TOL_F32
        assert rel_max(got, S_exact) <= TOL_F32
    else:
        assert rel_fro(got, S_exact) <= TOL_BF16
        assert rel_fro(got, S_exact) <= TOL_BF16_STORE
        assert_bf16_store_matches(to_host_bits(S), S_exact, S_store, "compress")


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
@pytest.mark.parametrize("d", [8, 64, 256, 12, 24, 344, 1032, 172, 20, 43, 86, 250])
def test_compress_gather_is_bit_exact(vl, dtype, d):
    # v = e_j: compress degenerates to a gather, so the indexing (group) is
    # checked with no rounding at all.
    N, M = (136 if d in (43, 86, 250) else 131), 5     # 136: X is a whole number of 16-byte vectors (LDS-tile kernel)
    D = M * d
    X = wl.random_tensor(N, D, dtype, seed=99)
    for j in (0, d // 2, d - 1):
        v = np.zeros(d, dtype=np.float32)
        v[j] = 1.0
        S = vl.velora_compress(to_dev(X, dtype), to_dev(v, wl.F32), M)
        want = X.reshape(N, M, d)[:, :, j]
        assert (to_host_bits(S) == want).all()


def test_compress_unaligned_views_take_generic_path(vl):
    torch = _torch()
    N, D, d = 64, 256, 64
    X = wl.random_tensor(N + 1, D, wl.BF16, seed=5)
    v = wl.random_unit_v(d, seed=1)
    Xd = to_dev(X, wl.BF16).reshape(-1)
    Xv = Xd[1:1 + N * D].view(N, D)                 # 2-byte aligned only
    assert Xv.data_ptr() % 16 != 0 and Xv.is_contiguous()
    S = vl.velora_compress(Xv, to_dev(v, wl.F32), D // d)
    Xh = np.ascontiguousarray(X.reshape(-1)[1:1 + N * D].reshape(N, D))
    S_exact, S_store = oracle.compress(Xh, v, D // d)
    assert_bf16_store_matches(to_host_bits(S), S_exact, S_store, "compress (unaligned)")
    torch.cuda.synchronize()


# ------------------------------------------------------------------ reconstruct
@pytest.mark.parametrize("N,D,d,dtype", [
    (256, 64, 16, wl.F32), (33, 96, 32, wl.BF16), (100, 768, 64, wl.BF16), (7, 60, 12, wl.BF16),
    (9, 63, 7, wl.F32), (5, 33, 1, wl.F32), (3, 2048, 1024, wl.BF16),
    # vectors that straddle sub-tokens (d not a multiple of the vector width, Xhat a whole number of vectors)
    (300, 11008, 43, wl.BF16), (150, 13824, 54, wl.BF16), (64, 24, 3, wl.BF16), (8, 9, 9, wl.BF16), (2048, 8, 1, wl.BF16),
    (300, 2752, 43, wl.F32), (4, 63, 7, wl.F32), (16, 20, 2, wl.F32), (40, 12000, 6000, wl.BF16),
])
def test_reconstruct_matches_oracle(vl, N, D, d, dtype):
    M = D // d
    S = wl.random_tensor(N, M, dtype, seed=3 + N)
    v = wl.random_unit_v(d, seed=2 + d)
    Xhat = vl.velora_reconstruct(to_dev(S, dtype), to_dev(v, wl.F32), D)
    want = oracle.reconstruct(S, v, D)
    got = to_host_f64(Xhat)
    if dtype == wl.F32:
        # one float32 multiply per element
        assert np.abs(got - want).max() <= 2.0 ** -23 * np.abs(want).max()
    else:
        assert rel_fro(got, want) <= TOL_BF16_STORE
        assert (np.abs(got - want) <= 2.0 ** -8 * np.abs(want) + 1e-30).all()


def test_projection_is_idempotent_on_gpu(vl):
    # compress(reconstruct(S)) = S |v|^2, through the HIP path alone
    N, D, d = 200, 256, 32
    S0 = wl.random_tensor(N, D // d, wl.F32, seed=8)
    v = wl.random_unit_v(d, seed=8)
    vd, Sd = to_dev(v, wl.F32), to_dev(S0, wl.F32)
    S1 = vl.velora_compress(vl.velora_reconstruct(Sd, vd, D), vd, D // d)
    np.testing.assert_allclose(to_host_f64(S1), S0.astype(np.float64), rtol=0, atol=2e-6 * np.abs(S0).max())


# ------------------------------------------------------------------ init_v
@pytest.mark.parametrize("N,D,d,dtype", [
    (256, 64, 16, wl.F32), (4 * 197, 768, 64, wl.BF16), (1000, 768, 128, wl.BF16), (555, 1024, 256, wl.BF16),
    (300, 2048, 1024, wl.BF16), (64, 4096, 2048, wl.BF16), (513, 96, 8, wl.F32), (100, 60, 12, wl.BF16),
    (77, 63, 7, wl.F32), (40, 33, 1, wl.F32), (3, 3000, 3000, wl.BF16),
    (700, 72, 24, wl.BF16), (333, 3 * 344, 344, wl.BF16), (210, 2 * 344, 344, wl.F32), (90, 2 * 1032, 1032, wl.BF16),
    (64, 2040, 2040, wl.BF16),
    # sub-token sizes the vector kernel cannot take, X a whole number of 16-byte vectors: column sums from LDS tiles
    (300, 11008, 43, wl.BF16), (150, 11008, 86, wl.BF16), (96, 13824, 54, wl.BF16), (64, 24, 3, wl.BF16),
    (8, 2 * 250, 250, wl.BF16), (300, 2752, 43, wl.F32), (52, 300, 100, wl.F32), (2048, 8, 1, wl.BF16), (5000, 86, 43, wl.BF16),
])
def test_init_v_matches_oracle(vl, N, D, d, dtype):
    M = D // d
    # a non-zero mean so that v is well conditioned (a zero-mean batch makes v a
    # normalised noise vector: still defined, tested at full size below)
    X32 = wl.random_tensor(N, D, wl.F32, seed=N + d).astype(np.float32)
    shift = np.tile(np.linspace(-1.0, 2.0, d, dtype=np.float32), M)
    X = wl.to_storage(X32 + shift[None, :], dtype)
    v = vl.velora_init_v(to_dev(X, dtype), M)
    v_ref, _, rc = oracle.init_v(X, M)
    assert rc == 0
    got = v.cpu().numpy().astype(np.float64)
    assert np.linalg.norm(got - v_ref.astype(np.float64)) <= 1e-5
    assert abs(np.linalg.norm(got) - 1.0) <= 1e-6


def test_init_v_degenerate(vl):
    torch = _torch()
    X = torch.zeros((64, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(vl.VeloraError) as ei:
        vl.velora_init_v(X, 4)
    assert ei.value.status == 6
    v = vl.velora_init_v(X, 4, allow_degenerate=True)
    assert (v.cpu().numpy() == np.float32(1.0 / np.sqrt(32.0))).all()
    Xn = torch.ones((64, 128), dtype=torch.float32, device="cuda")
    Xn[3, 5] = float("inf")
    v = vl.velora_init_v(Xn, 4, allow_degenerate=True)
    assert (v.cpu().numpy() == np.float32(1.0 / np.sqrt(32.0))).all()


# ------------------------------------------------------------------ per-batch v
@pytest.mark.parametrize("N,D,d,dtype", [
    (4 * 197, 768, 64, wl.BF16), (600, 1024, 256, wl.BF16), (300, 2048, 1024, wl.BF16), (513, 96, 8, wl.F32),
    (256, 64, 16, wl.F32), (100, 60, 12, wl.BF16), (77, 63, 7, wl.F32),
    (400, 72, 24, wl.BF16), (333, 3 * 344, 344, wl.BF16), (210, 2 * 344, 344, wl.F32), (90, 2 * 1032, 1032, wl.BF16),
])
def test_update_v_and_fused_compress_update(vl, N, D, d, dtype):
    torch = _torch()
    M = D // d
    beta = 0.75
    batches = []
    for i in range(3):
        X32 = wl.random_tensor(N, D, wl.F32, seed=100 * i + d).astype(np.float32)
        shift = np.tile(np.linspace(-1.0, 2.0, d, dtype=np.float32), M) * np.float32(1 + i)
        batches.append(wl.to_storage(X32 + shift[None, :], dtype))
    # --- velora_update_v chained over three batches against the oracle chain
    state_ref = np.zeros(d, dtype=np.float32)
    state = torch.zeros(d, dtype=torch.float32, device="cuda")
    for X in batches:
        v = vl.velora_update_v(to_dev(X, dtype), M, mean_state=state, beta=beta)
        v_ref, state_ref, rc = oracle.update_v(X, M, state=state_ref, beta=beta)
        assert rc == 0
        assert np.linalg.norm(v.cpu().numpy().astype(np.float64) - v_ref) <= 1e-5
        np.testing.assert_allclose(state.cpu().numpy(), state_ref, rtol=2e-6, atol=1e-6)
    # instance-wise: no state
    v_i = vl.velora_update_v(to_dev(batches[1], dtype), M)
    v_i_ref, _, _ = oracle.init_v(batches[1], M)
    assert np.linalg.norm(v_i.cpu().numpy().astype(np.float64) - v_i_ref) <= 1e-5
    # --- one pass: compress with the vector of the batches before, update for the next
    state_ref = np.zeros(d, dtype=np.float32)
    state = torch.zeros(d, dtype=torch.float32, device="cuda")
    v_cur_ref, _, _ = oracle.init_v(batches[0], M)                 # first batch: fixed-average start
    v_cur = to_dev(v_cur_ref, wl.F32)
    for X in batches:
        Xd = to_dev(X, dtype)
        S_plain = vl.velora_compress(Xd, v_cur, M)
        S, v_next = vl.velora_compress_update(Xd, v_cur, M, mean_state=state, beta=beta)
        assert torch.equal(S.view(torch.int16 if dtype == wl.BF16 else torch.int32),
                           S_plain.view(torch.int16 if dtype == wl.BF16 else torch.int32))
        S_exact, S_store = oracle.compress(X, v_cur.cpu().numpy(), M)
        assert rel_fro(to_host_f64(S), S_exact) <= (TOL_F32 if dtype == wl.F32 else TOL_BF16_STORE)
        v_next_ref, state_ref, _ = oracle.update_v(X, M, state=state_ref, beta=beta)
        assert np.linalg.norm(v_next.cpu().numpy().astype(np.float64) - v_next_ref) <= 1e-5
        v_cur = v_next


def test_update_v_degenerate_status_word(vl):
    torch = _torch()
    X = torch.zeros((64, 128), dtype=torch.bfloat16, device="cuda")
    need = vl.velora_workspace_bytes(vl.OP_INIT_V, 64, 128, 0, 4, vl.BF16)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    v = vl.velora_update_v(X, 4, ws=ws)
    torch.cuda.synchronize()
    assert int(ws[:4].view(torch.int32).item()) == 6
    assert (v.cpu().numpy() == np.float32(1.0 / np.sqrt(32.0))).all()


# ------------------------------------------------------------------ weight_grad
WGRAD_CASES = [
    # (N, O, D, d, dtype)
    (256, 64, 64, 16, wl.F32),                 # configuration 1
    (100, 50, 24, 3, wl.F32), (333, 70, 40, 40, wl.F32), (64, 9, 12, 1, wl.F32),
    # float32 inputs with O % 4 == 0 take the float32 matrix instruction: one, two and three group tiles, more
    # groups than one block covers (M = 100: three chunks), partial feature tiles, token counts around the
    # 16-token steps and the four waves' turns
    (515, 260, 2048, 128, wl.F32), (77, 520, 1024, 32, wl.F32), (300, 136, 1376, 32, wl.F32),    # M = 16, 32, 43
    (200, 128, 3200, 32, wl.F32), (1000, 64, 96, 32, wl.F32), (33, 12, 64, 16, wl.F32),          # M = 100, 3, 4
    (15, 4, 8, 8, wl.F32), (16, 132, 48, 1, wl.F32), (65, 8, 640, 2, wl.F32), (129, 36, 170, 10, wl.F32),   # M = 1, 48, 320, 17
    (4096, 512, 1376, 32, wl.F32),
    # bf16 MFMA tilings: M = D/d picks (S columns per lane, sets); O picks the G tile
    (1000, 256, 768, 64, wl.BF16),             # M = 12
    (777, 384, 768, 128, wl.BF16),             # M = 6, ragged token tail
    (515, 136, 2048, 128, wl.BF16),            # M = 16, partial O tile (136 = 128 + 8)
    (600, 128, 5120, 256, wl.BF16),            # M = 20
    (450, 72, 1376, 32, wl.BF16),              # M = 43 (odd: 2-byte S loads)
    (500, 96, 1728, 32, wl.BF16),              # M = 54
    (400, 64, 864, 32, wl.BF16),               # M = 27
    (520, 120, 5120, 64, wl.BF16),             # M = 80
    (300, 64, 1728, 8, wl.BF16),               # M = 216
    (260, 44, 640, 8, wl.BF16),                # M = 80, O % 8 != 0 -> 8-byte G loads
    (200, 36, 2400, 8, wl.BF16),               # M = 300 -> two group chunks
    (150, 30, 64, 16, wl.BF16),                # O % 4 != 0 -> generic kernel
    (130, 32, 40, 1, wl.BF16),                 # d = 1: dW = G^T S
    (90, 48, 512, 512, wl.BF16),               # M = 1: rank-one gradient
    (1, 16, 64, 16, wl.BF16), (31, 8, 16, 8, wl.BF16),
    # sub-token sizes that are not a multiple of four, float32 dW: four columns per store across group boundaries
    # (D % 4 == 0, d >= 4), several chunks of groups per row (M = 300 with many token ranges), and the scalar
    # rest (D % 4 != 0, d < 4)
    (300, 72, 11008, 43, wl.BF16), (200, 64, 86 * 16, 86, wl.BF16), (150, 40, 54 * 8, 54, wl.BF16),
    (120, 20, 36, 9, wl.BF16), (4000, 8, 1500, 5, wl.BF16), (90, 36, 35, 5, wl.BF16), (70, 12, 24, 3, wl.BF16),
    (257, 24, 43 * 12, 43, wl.F32),
    # two and three group tiles take the kernel whose loader waves stage G and S in LDS: token counts around
    # its 128-token chunks (127, 128, 129, one short of and one past several chunks per split), output widths
    # around its 128-feature tiles, group counts at both ends of each tile count, an odd N * M (falls back to
    # the per-wave kernel), and enough tokens that every split walks the three-slot ring more than once
    (127, 128, 544, 32, wl.BF16), (128, 8, 1024, 32, wl.BF16), (129, 136, 1056, 32, wl.BF16),   # M = 17, 32, 33
    (2, 264, 1536, 32, wl.BF16),                 # M = 48, two tokens
    (383, 120, 704, 16, wl.BF16),                # M = 44, odd N, even N * M
    (385, 128, 752, 16, wl.BF16),                # M = 47, N * M odd
    (40000, 128, 272, 16, wl.BF16),              # M = 17: 313 chunks, more than two per split
    (33000, 256, 1376, 32, wl.BF16),             # M = 43, ragged last chunk
    # up to five tiles on wide outputs (here: more than 8192 features) run on 256-feature blocks: output widths around
    # that tile, one that is not a multiple of 8 (per-wave kernel on the same token ranges), and a long
    # token axis (tens of chunks per block)
    (300, 8456, 512, 32, wl.BF16), (500, 8200, 320, 64, wl.BF16), (257, 8260, 256, 32, wl.BF16),   # M = 16, 5, 8
    (700, 8456, 1696, 32, wl.BF16), (600, 8200, 2560, 32, wl.BF16), (300, 8260, 2048, 32, wl.BF16),   # M = 53, 80, 64
    (450, 8448, 2080, 32, wl.BF16),              # M = 65
    (1, 8448, 512, 32, wl.BF16), (65, 8200, 96, 32, wl.BF16),   # one token; M = 3 and one token past a chunk
    # (up to three tiles: from 5377 output features on)
    (300, 5640, 1376, 32, wl.BF16), (500, 6152, 512, 32, wl.BF16), (200, 7176, 1024, 32, wl.BF16),   # M = 43, 16, 32
    (400, 6144, 2048, 32, wl.BF16),              # M = 64 at this width: 128-feature tiles
    (300, 8456, 1376, 32, wl.BF16), (1000, 8448, 640, 32, wl.BF16), (200, 8440, 1024, 32, wl.BF16),   # M = 43, 20, 32
    (310, 8260, 768, 32, wl.BF16),               # M = 24, O % 8 != 0
    (8000, 8200, 544, 32, wl.BF16),              # M = 17
    # four group tiles: the loader-wave kernel with 64-token chunks and the features split over two waves
    (63, 128, 1568, 32, wl.BF16), (64, 72, 2048, 32, wl.BF16), (65, 264, 2016, 32, wl.BF16),   # M = 49, 64, 63
    (1000, 136, 416, 8, wl.BF16),                # M = 52
    (30000, 128, 512, 8, wl.BF16),               # M = 64: many chunks per split
    # five and six group tiles in the same kernel (all blocks resident at once)
    (64, 64, 1040, 16, wl.BF16), (700, 128, 1520, 16, wl.BF16), (333, 200, 1536, 16, wl.BF16),   # M = 65, 95, 96
    (9000, 256, 640, 8, wl.BF16),                # M = 80: several chunks per split
]


@pytest.mark.parametrize("N,O,D,d,dtype", WGRAD_CASES)
def test_weight_grad_matches_bruteforce_oracle(vl, N, O, D, d, dtype):
    M = D // d
    G = wl.random_tensor(N, O, dtype, seed=N + O, stream=7, sigma=0.02)
    S = wl.random_tensor(N, M, dtype, seed=N + M, stream=8)
    v = wl.random_unit_v(d, seed=d + 1)
    dW = vl.velora_weight_grad(to_dev(G, dtype), to_dev(S, dtype), to_dev(v, wl.F32), D)
    want = oracle.weight_grad_bruteforce(G, S, v, D)
    got = to_host_f64(dW)
    assert got.shape == (O, D)
    if dtype == wl.F32:
        assert rel_fro(got, want) <= TOL_F32
        assert rel_max(got, want) <= TOL_F32
    else:
        assert rel_fro(got, want) <= TOL_BF16
        assert rel_fro(got, want) <= TOL_F32_FROM_BF16
        assert rel_max(got, want) <= TOL_F32_FROM_BF16


@pytest.mark.parametrize("N,O,D,d", [(515, 136, 2048, 128), (300, 64, 1728, 8), (150, 30, 64, 16), (200, 24, 43 * 8, 43)])
def test_weight_grad_bf16_output_and_accumulate(vl, N, O, D, d):
    torch = _torch()
    M = D // d
    G = wl.random_tensor(N, O, wl.BF16, seed=1, stream=7, sigma=0.02)
    S = wl.random_tensor(N, M, wl.BF16, seed=2, stream=8)
    v = wl.random_unit_v(d, seed=3)
    Gd, Sd, vd = to_dev(G, wl.BF16), to_dev(S, wl.BF16), to_dev(v, wl.F32)
    want = oracle.weight_grad_bruteforce(G, S, v, D)
    # bf16 output: one extra rounding
    dWb = vl.velora_weight_grad(Gd, Sd, vd, D, dw_dtype=torch.bfloat16)
    assert dWb.dtype == torch.bfloat16
    assert rel_fro(to_host_f64(dWb), want) <= TOL_BF16_STORE
    # accumulate into an existing float32 gradient
    base = wl.random_tensor(O, D, wl.F32, seed=4, sigma=0.5)
    dW = to_dev(base, wl.F32)
    vl.velora_weight_grad(Gd, Sd, vd, D, dW=dW, accumulate=True)
    assert rel_fro(to_host_f64(dW), base.astype(np.float64) + want) <= TOL_F32_FROM_BF16
    # accumulate into bf16
    baseb = wl.random_tensor(O, D, wl.BF16, seed=5, sigma=0.5)
    dWa = to_dev(baseb, wl.BF16)
    vl.velora_weight_grad(Gd, Sd, vd, D, dW=dWa, accumulate=True)
    assert rel_fro(to_host_f64(dWa), wl.to_f64(baseb, wl.BF16) + want) <= TOL_BF16_STORE


# Rows of dW of 32 KB and more are written by the window-sweep kernel: one sweep of the whole grid over dW
# with a per-block table of T.  Cases: fewer blocks than compute units (a multiple of eight and not), a
# sub-token of 43 or 86 vectors (table positions drift from window to window), 16 vectors (the smallest the
# kernel takes) and 512, a ragged last trip, more than eight token ranges, bf16 dW in 16-byte and 8-byte
# vectors, accumulation, and the hand-off entry points on the same shapes.
LONG_ROW_CASES = [
    # (N, O, D, d, dW dtype)
    (300, 8, 8192, 64, "f32"), (300, 5, 8256, 172, "f32"), (200, 3, 16384, 1024, "f32"),
    (2000, 300, 8192, 2048, "f32"), (700, 131, 11008, 344, "f32"), (8192, 2048, 8192, 256, "f32"),
    (300, 8, 16384, 128, "bf16"), (260, 12, 16512, 172, "bf16"), (1500, 260, 16384, 256, "bf16"),
    # bf16 output takes the sweep at every row length (sub-tokens of 128 elements and more)
    (400, 70, 11008, 256, "bf16"), (250, 33, 10752, 128, "bf16"), (300, 20, 13824, 256, "bf16"),
    (200, 40, 1024, 128, "bf16"), (129, 7, 768, 128, "bf16"), (90, 1, 256, 256, "bf16"), (500, 300, 4096, 1024, "bf16"),
]


@pytest.mark.parametrize("N,O,D,d,dw", LONG_ROW_CASES)
def test_weight_grad_long_rows(vl, N, O, D, d, dw):
    torch = _torch()
    M = D // d
    G = wl.random_tensor(N, O, wl.BF16, seed=N + O + 11, stream=7, sigma=0.02)
    S = wl.random_tensor(N, M, wl.BF16, seed=N + M + 12, stream=8)
    v = wl.random_unit_v(d, seed=d + 5)
    Gd, Sd, vd = to_dev(G, wl.BF16), to_dev(S, wl.BF16), to_dev(v, wl.F32)
    T_ref, want = oracle.weight_grad_factored(G, S, v, D)
    tdt = torch.float32 if dw == "f32" else torch.bfloat16
    tol = TOL_F32_FROM_BF16 if dw == "f32" else TOL_BF16_STORE
    dW = vl.velora_weight_grad(Gd, Sd, vd, D, dw_dtype=tdt)
    got = to_host_f64(dW)
    assert got.shape == (O, D)
    assert rel_fro(got, want) <= tol
    if dw == "f32":
        assert rel_max(got, want) <= tol
    # every row on its own (a misplaced table entry would spoil single rows, not the norm of the whole)
    row_err = np.linalg.norm(got - want, axis=1) / (np.linalg.norm(want, axis=1) + 1e-300)
    assert row_err.max() <= 4 * tol
    # accumulate into an existing gradient of the same dtype
    if dw == "f32":
        base = wl.random_tensor(O, D, wl.F32, seed=4, sigma=0.5)
        acc = to_dev(base, wl.F32)
        base64 = base.astype(np.float64)
    else:
        base = wl.random_tensor(O, D, wl.BF16, seed=5, sigma=0.5)
        acc = to_dev(base, wl.BF16)
        base64 = wl.to_f64(base, wl.BF16)
    vl.velora_weight_grad(Gd, Sd, vd, D, dW=acc, accumulate=True)
    assert rel_fro(to_host_f64(acc), base64 + want) <= tol
    # the hand-off: expanding an exactly known T is one float32 multiply per element
    if dw == "f32":
        T1 = (torch.arange(O * M, dtype=torch.float32, device="cuda").reshape(O, M) % 1021.0) - 7.0
        dW1 = vl.velora_expand_factor(T1, vd, D).cpu().numpy().reshape(O, M, d)
        assert (dW1 == T1.cpu().numpy()[:, :, None] * v[None, None, :]).all()


@pytest.mark.parametrize("N,O,D,d,dtype", [
    (256, 64, 64, 16, wl.F32), (1000, 256, 768, 64, wl.BF16), (450, 72, 1376, 32, wl.BF16),
    (520, 120, 5120, 64, wl.BF16), (300, 64, 1728, 8, wl.BF16), (150, 30, 64, 16, wl.BF16),
])
def test_factored_handoff(vl, N, O, D, d, dtype):
    # T = G^T S on its own, its expansion, and their agreement with weight_grad
    torch = _torch()
    M = D // d
    G = wl.random_tensor(N, O, dtype, seed=N + 3, stream=7, sigma=0.02)
    S = wl.random_tensor(N, M, dtype, seed=N + 4, stream=8)
    v = wl.random_unit_v(d, seed=d + 2)
    Gd, Sd, vd = to_dev(G, dtype), to_dev(S, dtype), to_dev(v, wl.F32)
    T = vl.velora_weight_grad_factor(Gd, Sd)
    T_ref, dW_ref = oracle.weight_grad_factored(G, S, v, D)
    tol = TOL_F32 if dtype == wl.F32 else TOL_F32_FROM_BF16
    assert T.shape == (O, M) and T.dtype == torch.float32
    assert rel_fro(to_host_f64(T), T_ref) <= tol and rel_max(to_host_f64(T), T_ref) <= tol
    dW = vl.velora_expand_factor(T, vd, D)
    assert rel_fro(to_host_f64(dW), dW_ref) <= tol
    # weight_grad is factor followed by expand (the token split may differ, so not bit for bit)
    dW2 = vl.velora_weight_grad(Gd, Sd, vd, D)
    assert rel_fro(to_host_f64(dW), to_host_f64(dW2)) <= 2e-6
    # expanding an exactly known T: one float32 multiply per element
    T1 = torch.arange(O * M, dtype=torch.float32, device="cuda").reshape(O, M) - 7.0
    dW1 = vl.velora_expand_factor(T1, vd, D).cpu().numpy().reshape(O, M, d)
    want = T1.cpu().numpy()[:, :, None] * v[None, None, :]
    assert (dW1 == want).all()


def test_weight_grad_single_one_copies_reconstructed_token(vl):
    # G = e_n e_o^T: row o of dW is the reconstructed token n, everything else 0.
    N, O, D, d = 160, 128, 256, 32
    M = D // d
    S = wl.random_tensor(N, M, wl.BF16, seed=12)
    v = wl.random_unit_v(d, seed=12)
    Xhat = oracle.reconstruct(S, v, D)
    for (n, o) in [(0, 0), (159, 127), (77, 5), (31, 64), (32, 63)]:
        G = np.zeros((N, O), dtype=np.uint16)
        G[n, o] = 0x3F80                                    # 1.0 in bf16
        dW = to_host_f64(vl.velora_weight_grad(to_dev(G, wl.BF16), to_dev(S, wl.BF16), to_dev(v, wl.F32), D))
        np.testing.assert_allclose(dW[o], Xhat[n], rtol=2e-7, atol=0)
        mask = np.ones(O, dtype=bool)
        mask[o] = False
        assert (dW[mask] == 0).all()


def test_weight_grad_is_deterministic(vl):
    N, O, D, d = 2048, 256, 1024, 64
    G = wl.random_tensor(N, O, wl.BF16, seed=21, sigma=0.02)
    S = wl.random_tensor(N, D // d, wl.BF16, seed=22)
    v = wl.random_unit_v(d, seed=23)
    Gd, Sd, vd = to_dev(G, wl.BF16), to_dev(S, wl.BF16), to_dev(v, wl.F32)
    a = vl.velora_weight_grad(Gd, Sd, vd, D).cpu().numpy()
    for _ in range(3):
        b = vl.velora_weight_grad(Gd, Sd, vd, D).cpu().numpy()
        assert (a.view(np.uint32) == b.view(np.uint32)).all()


def test_end_to_end_config1(vl):
    # BASELINE configuration 1 through the whole path: init_v -> compress -> weight_grad
    sh = wl.shape_by_name("cfg1_tiny")
    X, G = wl.make_X(sh), wl.make_G(sh)
    Xd, Gd = to_dev(X, sh.dtype), to_dev(G, sh.dtype)
    v = vl.velora_init_v(Xd, sh.M)
    S = vl.velora_compress(Xd, v, sh.M)
    dW = vl.velora_weight_grad(Gd, S, v, sh.D)
    v_ref, _, _ = oracle.init_v(X, sh.M)
    S_exact, S_store = oracle.compress(X, v_ref, sh.M)
    want = oracle.weight_grad_bruteforce(G, S_store, v_ref, sh.D)
    assert np.linalg.norm(v.cpu().numpy().astype(np.float64) - v_ref) <= 1e-5
    assert rel_fro(to_host_f64(S), S_exact) <= TOL_F32
    assert rel_fro(to_host_f64(dW), want) <= TOL_F32
    assert rel_max(to_host_f64(dW), want) <= TOL_F32


def test_shape_error_reaches_python(vl):
    torch = _torch()
    X = torch.zeros((4, 13824), dtype=torch.bfloat16, device="cuda")
    v = torch.zeros(1024, dtype=torch.float32, device="cuda")
    with pytest.raises(vl.VeloraError) as ei:
        vl.velora_compress(X, v, 13)                        # 13824 / 1024 is not an integer
    assert ei.value.status == 2


@pytest.mark.parametrize("nbytes", [16, 4096 + 16, (3 << 20) + 48, 64 << 20])
def test_bandwidth_probe_kernels_move_what_they_claim(vl, nbytes):
    # the streaming probes that bench.py's measured ceilings come from: copy is bit-exact and touches nothing
    # past the end, write leaves zeros, read leaves its source alone
    torch = _torch()
    g = torch.Generator(device="cuda").manual_seed(nbytes % 9973)
    src = torch.randint(0, 256, (nbytes + 64,), dtype=torch.uint8, device="cuda", generator=g)
    keep = src.clone()
    dst = torch.full((nbytes + 64,), 0xAB, dtype=torch.uint8, device="cuda")
    vl.velora_bandwidth_probe("copy", src=src[:nbytes], dst=dst[:nbytes])
    assert torch.equal(dst[:nbytes], src[:nbytes]) and bool((dst[nbytes:] == 0xAB).all())
    vl.velora_bandwidth_probe("write", dst=dst[:nbytes])
    assert int(dst[:nbytes].count_nonzero()) == 0 and bool((dst[nbytes:] == 0xAB).all())
    sink = torch.zeros(64, dtype=torch.int32, device="cuda")
    vl.velora_bandwidth_probe("read", src=src[:nbytes], sink=sink)
    torch.cuda.synchronize()
    assert torch.equal(src, keep)
