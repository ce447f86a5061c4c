"""GPU parity past 2^31 elements: X[N, D] and G[N, O] each hold more than 2^31 values, so any
32-bit element index in the kernels or in the launch arithmetic would wrap.  Inputs are seeded and
drawn on the device (4.3 GB each; the host generator would take minutes), their bits are copied
to the host and the oracle works from exactly those bits."""
import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_helpers import TOL_BF16_STORE, TOL_F32_FROM_BF16, rel_fro, to_host_bits, to_host_f64

pytestmark = pytest.mark.gpu

N = (1 << 21) + 77          # ragged: not a multiple of any tile
D = 1024
O = 1032                    # N*O > 2^31 as well; a multiple of 8 so the MFMA path is taken
M = 8                       # d = 128


@pytest.fixture(scope="module")
def vl():
    import __graft_entry__ as ge
    ge.ensure_built()
    import paper_2405_17991_amd as vl
    return vl


def test_more_than_2_31_elements(vl):
    import torch
    assert N * D > 2**31 and N * O > 2**31
    g = torch.Generator(device="cuda")
    g.manual_seed(20240531)
    X = torch.empty((N, D), device="cuda", dtype=torch.bfloat16)
    step = 1 << 18
    for r0 in range(0, N, step):                      # in slabs: the float32 draw of the whole array would be 8.6 GB
        r1 = min(N, r0 + step)
        X[r0:r1] = (torch.randn((r1 - r0, D), generator=g, device="cuda") + 0.25).to(torch.bfloat16)
    G = torch.empty((N, O), device="cuda", dtype=torch.bfloat16)
    for r0 in range(0, N, step):
        r1 = min(N, r0 + step)
        G[r0:r1] = (torch.randn((r1 - r0, O), generator=g, device="cuda") * 0.01).to(torch.bfloat16)
    torch.cuda.synchronize()
    print(f"\n[large] N={N} D={D} O={O} M={M}: inputs on device", flush=True)

    # ---- init_v over all 2.2e9 elements
    Xh = to_host_bits(X)
    v_gpu = vl.velora_init_v(X, M)
    v_ref, _, rc = oracle.init_v(Xh, M)
    assert rc == 0
    err_v = float(np.linalg.norm(v_gpu.cpu().numpy().astype(np.float64) - v_ref.astype(np.float64)))
    print(f"  init_v |dv| = {err_v:.2e}", flush=True)
    assert err_v <= 1e-5

    # ---- compress: every output, with the oracle's v
    vd = torch.from_numpy(v_ref).cuda()
    S = vl.velora_compress(X, vd, M)
    torch.cuda.synchronize()
    S_exact, S_store = oracle.compress(Xh, v_ref, M)
    r = rel_fro(to_host_f64(S), S_exact)
    print(f"  compress rel_fro = {r:.2e}", flush=True)
    assert r <= TOL_BF16_STORE
    got_bits = to_host_bits(S)
    # the rows whose flat element offsets straddle 2^31 and the very last rows, bit for bit up to 1 ulp
    for row in (0, (2**31) // D - 1, (2**31) // D, (2**31) // D + 1, N - 2, N - 1):
        d = np.abs(got_bits[row].astype(np.int32) - S_store[row].astype(np.int32))
        assert d.max() <= 1, (row, got_bits[row], S_store[row])
    del X, Xh, S_exact
    torch.cuda.empty_cache()

    # ---- weight_grad from the oracle's stored S; sampled output rows from the definition
    Sd = torch.from_numpy(S_store).view(torch.bfloat16).cuda()
    dW = vl.velora_weight_grad(G, Sd, vd, D)
    torch.cuda.synchronize()
    Gh = to_host_bits(G)
    rows = [0, 1, 127, 128, 515, O - 9, O - 8, O - 1]
    ref = oracle.weight_grad_bruteforce_rows(Gh, S_store, v_ref, D, rows)
    got = dW[rows].cpu().numpy().astype(np.float64)
    r = rel_fro(got, ref)
    print(f"  weight_grad rel_fro on {len(rows)} rows = {r:.2e}", flush=True)
    assert r <= TOL_F32_FROM_BF16
    # and the factor route agrees with it everywhere
    T = vl.velora_weight_grad_factor(G, Sd)
    dW2 = vl.velora_expand_factor(T, vd, D)
    torch.cuda.synchronize()
    assert rel_fro(dW2.cpu().numpy().astype(np.float64), dW.cpu().numpy().astype(np.float64)) <= 2e-6


def test_dense_products_past_2_31_elements(vl):
    """velora_linear_compress and velora_grad_input with X (and dX) beyond 2^31 elements: the row
    offsets of the last token tiles do not fit 32 bits.  Rows on both sides of the 2^31 boundary
    and the last rows are checked against the oracle's per-row products."""
    import torch
    from gpu_helpers import assert_bf16_store_matches
    Ox = 264
    g = torch.Generator(device="cuda")
    g.manual_seed(77)
    X = torch.empty((N, D), device="cuda", dtype=torch.bfloat16)
    step = 1 << 18
    for r0 in range(0, N, step):
        r1 = min(N, r0 + step)
        X[r0:r1] = torch.randn((r1 - r0, D), generator=g, device="cuda").to(torch.bfloat16)
    W = (torch.randn((Ox, D), generator=g, device="cuda") * D ** -0.5).to(torch.bfloat16)
    v = wl.random_unit_v(D // M, seed=5)
    vd = torch.from_numpy(v).cuda()
    Y, S = vl.velora_linear_compress(X, W, vd, M)
    torch.cuda.synchronize()
    rows = np.array([0, 255, 256, (2**31) // D - 1, (2**31) // D, (2**31) // D + 1, N - 78, N - 77, N - 1])
    idx = torch.from_numpy(rows).cuda()
    Y_exact, Y_store, S_exact, S_store = oracle.linear_compress(to_host_bits(X[idx]), to_host_bits(W), v, M)
    assert_bf16_store_matches(to_host_bits(Y[idx]), Y_exact, Y_store, "Y rows")
    assert_bf16_store_matches(to_host_bits(S[idx]), S_exact, S_store, "S rows")
    del Y, S
    # dX[N, D] = G[N, Ox] W[Ox, D]: the output is the array past 2^31 elements here (Ox % 64 != 0 would leave
    # the MFMA path, so the reduction length is cut to 256)
    Gx = (torch.randn((N, 256), generator=g, device="cuda") * 0.05).to(torch.bfloat16)
    W2 = W[:256].contiguous()
    dX = vl.velora_grad_input(Gx, W2)
    torch.cuda.synchronize()
    dX_exact, dX_store = oracle.grad_input(to_host_bits(Gx[idx]), to_host_bits(W2))
    assert_bf16_store_matches(to_host_bits(dX[idx]), dX_exact, dX_store, "dX rows")
