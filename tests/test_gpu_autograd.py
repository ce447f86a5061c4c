"""The autograd wrapper around the two VeLoRA kernels (paper Listing 1): the
forward output is the dense product, the weight gradient is the one built from
compressed activations, and what autograd keeps for backward shrinks by d."""
import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_helpers import TOL_BF16_STORE, TOL_F32, rel_fro, to_dev, to_host_bits, to_host_f64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mods():
    import __graft_entry__ as ge
    ge.ensure_built()
    import torch
    from paper_2405_17991_amd import autograd as va
    return torch, va


@pytest.mark.parametrize("dtype,B,T,D,O,d", [("bf16", 4, 197, 768, 256, 64), ("f32", 2, 128, 64, 48, 16)])
def test_layer_forward_backward(mods, dtype, B, T, D, O, d):
    torch, va = mods
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    sdt = wl.BF16 if dtype == "bf16" else wl.F32
    torch.manual_seed(0)
    layer = va.VeLoRALinear(D, O, d, device="cuda", dtype=tdt)
    Xh = wl.random_tensor(B * T, D, sdt, seed=7)
    Xh = wl.to_storage(wl.to_f64(Xh, sdt).astype(np.float32) + 0.5, sdt)      # non-zero mean: well-conditioned v
    Gh = wl.random_tensor(B * T, O, sdt, seed=8, sigma=0.02)
    x = to_dev(Xh, sdt).reshape(B, T, D).requires_grad_(True)
    out = layer(x)
    assert out.shape == (B, T, O) and bool(layer.v_ready)
    ref = torch.nn.functional.linear(x.detach(), layer.weight.detach())
    assert torch.equal(out.detach(), ref)                                      # the dense forward is untouched
    g = to_dev(Gh, sdt).reshape(B, T, O)
    out.backward(g)
    # v: the normalised mean of the first batch's sub-tokens
    v_ref, _, rc = oracle.init_v(Xh, D // d)
    assert rc == 0
    v_gpu = layer.v.cpu().numpy()
    assert np.linalg.norm(v_gpu.astype(np.float64) - v_ref) <= 1e-5
    # grad_weight = G^T Xhat with Xhat rebuilt from the stored S (oracle, from the definition)
    _, S_store = oracle.compress(Xh, v_gpu, D // d)
    want = oracle.weight_grad_bruteforce(Gh, S_store, v_gpu, D)
    got = to_host_f64(layer.weight.grad)
    assert got.shape == (O, D)
    assert rel_fro(got, want) <= (2 * TOL_BF16_STORE if dtype == "bf16" else 10 * TOL_F32)
    # grad_input is the untouched dense product
    gi = torch.matmul(g.reshape(-1, O), layer.weight.detach()).reshape(B, T, D)
    assert torch.equal(x.grad, gi)
    # v stays frozen on later batches
    before = layer.v.clone()
    layer(x.detach() * 3.0)
    assert torch.equal(layer.v, before)


def test_layer_with_the_package_s_own_gemms(mods):
    # the same layer with both dense products in this package's kernels: same forward and gradients as the
    # vendor-GEMM variant up to the rounding of bf16 outputs
    torch, va = mods
    torch.manual_seed(1)
    B, T, D, O, d = 3, 100, 256, 264, 64
    a = va.VeLoRALinear(D, O, d, device="cuda", dtype=torch.bfloat16)
    b = va.VeLoRALinear(D, O, d, device="cuda", dtype=torch.bfloat16, own_gemm=True)
    b.load_state_dict(a.state_dict())
    x = (torch.randn(B, T, D, device="cuda") + 0.5).to(torch.bfloat16)
    g = (torch.randn(B, T, O, device="cuda") * 0.05).to(torch.bfloat16)
    xa = x.clone().requires_grad_(True)
    xb = x.clone().requires_grad_(True)
    ya = a(xa); ya.backward(g)
    yb = b(xb); yb.backward(g)
    torch.cuda.synchronize()
    assert torch.equal(a.v, b.v)

    def rel(p, q):
        return ((p.float() - q.float()).norm() / q.float().norm()).item()

    assert rel(yb, ya) <= 4e-3 and rel(xb.grad, xa.grad) <= 4e-3 and rel(b.weight.grad, a.weight.grad) <= 4e-3


def test_saved_activation_shrinks_by_d(mods):
    torch, va = mods
    N, D, O, d = 2048, 1024, 512, 64
    layer = va.VeLoRALinear(D, O, d, device="cuda", dtype=torch.bfloat16)
    x = torch.randn(N, D, device="cuda", dtype=torch.bfloat16)
    layer.init_v(x)

    def saved_bytes(fn):
        seen = {}

        def pack(t):
            if t.data_ptr() not in (layer.weight.data_ptr(), layer.v.data_ptr()):
                seen[t.data_ptr()] = t.numel() * t.element_size()
            return t

        with torch.autograd.graph.saved_tensors_hooks(pack, lambda t: t):
            fn()
        return sum(seen.values())

    base = saved_bytes(lambda: torch.nn.functional.linear(x.requires_grad_(True), layer.weight))
    ours = saved_bytes(lambda: layer(x.requires_grad_(True)))
    acc = va.saved_activation_bytes(N, D, d, 2)
    assert base == acc["baseline"] == N * D * 2
    assert ours == acc["velora"] == N * (D // d) * 2
    assert base // ours == d


def test_device_memory_held_between_forward_and_backward(mods):
    # the allocator's view of the same claim, at a LLaMA-7B-like layer width: after the forward,
    # with the caller's own reference to the activation dropped, a plain linear keeps it alive
    # (N*D*2 bytes) while the VeLoRA layer keeps only S (N*D/d*2 bytes, up to allocator rounding)
    torch, va = mods
    N, D, O, d = 4096, 4096, 1024, 256
    layer = va.VeLoRALinear(D, O, d, device="cuda", dtype=torch.bfloat16)
    layer.init_v(torch.randn(N, D, device="cuda", dtype=torch.bfloat16))

    def held(fn):
        # the layer input is a non-leaf activation (as inside a network): once the caller drops
        # it, only what autograd saved keeps memory alive
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        leaf = torch.zeros(N, 1, device="cuda", dtype=torch.bfloat16, requires_grad=True)
        noise = torch.randn(N, D, device="cuda", dtype=torch.bfloat16)
        base = torch.cuda.memory_allocated()
        xin = noise + leaf                            # add saves nothing for its backward
        y = fn(xin)
        out_bytes = y.numel() * y.element_size()
        del xin
        torch.cuda.synchronize()
        kept = torch.cuda.memory_allocated() - base - out_bytes
        y.sum().backward()
        assert leaf.grad is not None
        return kept

    plain = held(lambda t: torch.nn.functional.linear(t, layer.weight))
    ours = held(lambda t: layer(t))
    assert plain >= N * D * 2                        # the input itself is still held for backward
    assert ours <= N * (D // d) * 2 + (2 << 20)      # only S (plus allocator block rounding)
    assert plain - ours >= N * D * 2 - N * (D // d) * 2 - (2 << 20)


def _reference_mlp_grads(torch, h, wg, wu, wd, v_h, v_f, gout):
    """The same block written with plain torch ops: dense forward, and for every weight
    the paper's backward rule grad_weight = grad_output^T @ reconstruct(compress(input))."""
    d_h, d_f = v_h.numel(), v_f.numel()

    def proj(x, v, d):       # reconstruct(compress(x)), S rounded to the storage dtype as the library stores it
        n, D = x.shape
        z = x.float().reshape(n, D // d, d)
        s = (z @ v).to(x.dtype).float()
        return (s.unsqueeze(-1) * v).reshape(n, D)

    hf = h.float()
    gate = (h @ wg.t()); up = (h @ wu.t())
    X = (torch.nn.functional.silu(gate.float()) * up.float()).to(h.dtype)
    out = X @ wd.t()
    go = gout.float()
    dWd = go.t() @ proj(X, v_f, d_f)
    dX = go @ wd.float()
    gf = gate.float(); sig = torch.sigmoid(gf)
    dup = (dX * gf * sig).to(h.dtype); dgate = (dX * up.float() * sig * (1 + gf * (1 - sig))).to(h.dtype)
    ph = proj(h, v_h, d_h)
    dWg = dgate.float().t() @ ph
    dWu = dup.float().t() @ ph
    dh = dgate.float() @ wg.float() + dup.float() @ wu.float()
    return out, dWg, dWu, dWd, dh


def test_llama_mlp_block_matches_the_same_rule_in_plain_torch(mods):
    torch, va = mods
    torch.manual_seed(3)
    N, H, F, d_h, d_f = 512, 256, 704, 64, 64
    blk = va.VeLoRALlamaMLP(H, F, d_h, d_f, device="cuda", dtype=torch.bfloat16)
    h = torch.randn(N, H, device="cuda", dtype=torch.bfloat16, requires_grad=True)
    gout = (torch.randn(N, H, device="cuda") * 0.05).to(torch.bfloat16)
    out = blk(h)
    out.backward(gout)
    torch.cuda.synchronize()
    ro, rg, ru, rd, rh = _reference_mlp_grads(torch, h.detach(), blk.w_gate.detach(), blk.w_up.detach(),
                                              blk.w_down.detach(), blk.v_h, blk.v_f, gout)

    def rel(a, b):
        return ((a.float() - b.float()).norm() / b.float().norm()).item()

    assert rel(out, ro) <= 2e-2
    assert rel(blk.w_gate.grad, rg) <= 2e-2 and rel(blk.w_up.grad, ru) <= 2e-2 and rel(blk.w_down.grad, rd) <= 2e-2
    assert rel(h.grad, rh) <= 2e-2


def test_llama_mlp_block_keeps_scalars_instead_of_inputs(mods):
    torch, va = mods
    N, H, F, d_h, d_f = 2048, 1024, 2816, 128, 128
    blk = va.VeLoRALlamaMLP(H, F, d_h, d_f, device="cuda", dtype=torch.bfloat16)
    blk.init_v(torch.randn(N, H, device="cuda", dtype=torch.bfloat16))
    params = {p.data_ptr() for p in blk.parameters()} | {blk.v_h.data_ptr(), blk.v_f.data_ptr()}
    seen = {}

    def pack(t):
        if t.data_ptr() not in params:
            seen[t.data_ptr()] = t.numel() * t.element_size()
        return t

    h = torch.randn(N, H, device="cuda", dtype=torch.bfloat16, requires_grad=True)
    with torch.autograd.graph.saved_tensors_hooks(pack, lambda t: t):
        blk(h)
    # gate and up (for the activation's backward) plus one scalar per sub-token of h and of the product;
    # neither h (N*H) nor the product (N*F) is kept
    assert sum(seen.values()) == 2 * N * F * 2 + N * (H // d_h) * 2 + N * (F // d_f) * 2


def test_norm_qkv_block_matches_the_same_rule_in_plain_torch(mods):
    torch, va = mods
    torch.manual_seed(5)
    N, H, d = 384, 512, 64
    blk = va.VeLoRANormLinears(H, (H, 256, 256), d, device="cuda", dtype=torch.bfloat16)
    with torch.no_grad():
        blk.gamma.copy_(torch.linspace(0.5, 1.5, H, device="cuda"))
    h = (torch.randn(N, H, device="cuda") + 0.3).to(torch.bfloat16).requires_grad_(True)
    gouts = [(torch.randn(N, o, device="cuda") * 0.05).to(torch.bfloat16) for o in (H, 256, 256)]
    outs = blk(h)
    torch.autograd.backward(outs, gouts)
    torch.cuda.synchronize()
    # the same rule with plain torch ops: dense forward, weight gradients from reconstruct(compress(X))
    hf = h.detach().float()
    rinv = torch.rsqrt(hf.pow(2).mean(-1, keepdim=True) + blk.eps)
    X = (hf * rinv * blk.gamma.detach()).to(torch.bfloat16)
    z = X.float().reshape(N, H // d, d)
    s = (z @ blk.v).to(torch.bfloat16).float()
    Xp = (s.unsqueeze(-1) * blk.v).reshape(N, H)

    def rel(a, b):
        return ((a.float() - b.float()).norm() / b.float().norm()).item()

    dX = torch.zeros(N, H, device="cuda")
    for o, w, g in zip(outs, blk.weights, gouts):
        assert rel(o, X @ w.detach().t()) <= 1e-2
        assert rel(w.grad, g.float().t() @ Xp) <= 2e-2
        dX += g.float() @ w.detach().float()
    xhat = hf * rinv
    dxg = dX * blk.gamma.detach()
    want_h = rinv * (dxg - xhat * (dxg * xhat).mean(-1, keepdim=True))
    assert rel(h.grad, want_h) <= 2e-2
    assert rel(blk.gamma.grad, (dX * xhat).sum(0)) <= 2e-2
    # and against autograd through torch's own rms_norm for the parts VeLoRA does not change
    h2 = h.detach().clone().requires_grad_(True)
    g2 = blk.gamma.detach().clone().requires_grad_(True)
    Xr = torch.nn.functional.rms_norm(h2.float(), (H,), g2, blk.eps).to(torch.bfloat16)
    torch.autograd.backward([Xr @ w.detach().t() for w in blk.weights], gouts)
    assert rel(h.grad, h2.grad) <= 2e-2 and rel(blk.gamma.grad, g2.grad) <= 2e-2


def test_norm_qkv_block_keeps_scalars_instead_of_the_normalised_input(mods):
    torch, va = mods
    N, H, d = 2048, 1024, 128
    blk = va.VeLoRANormLinears(H, (H, H, H), d, device="cuda", dtype=torch.bfloat16)
    blk.init_v(torch.randn(N, H, device="cuda", dtype=torch.bfloat16))
    params = {p.data_ptr() for p in blk.parameters()} | {blk.v.data_ptr()}
    seen = {}

    def pack(t):
        if t.data_ptr() not in params:
            seen[t.data_ptr()] = t.numel() * t.element_size()
        return t

    h = torch.randn(N, H, device="cuda", dtype=torch.bfloat16, requires_grad=True)
    with torch.autograd.graph.saved_tensors_hooks(pack, lambda t: t):
        blk(h)
    # h itself (for the normalisation's backward) and one scalar per sub-token; the normalised input is not kept
    assert sum(seen.values()) == N * H * 2 + N * (H // d) * 2


def test_v_flag_lives_on_the_host_and_follows_the_state_dict(mods):
    """forward never reads the device flag; loading a state dict that holds v marks the module ready; a
    module that has seen no training batch runs the plain layer in eval mode; a degenerate first batch warns
    and leaves the module waiting for the next batch."""
    torch, va = mods
    torch.manual_seed(1)
    a = va.VeLoRALinear(128, 64, 32, device="cuda", dtype=torch.bfloat16)
    x = (torch.randn((40, 128), device="cuda") + 0.5).to(torch.bfloat16)
    a.eval()
    y = a(x)                                              # eval before any training batch: plain layer, v untouched
    assert not a._v_ready_host and not bool(a.v_ready) and float(a.v.abs().sum()) == 0.0
    assert torch.equal(y, torch.nn.functional.linear(x, a.weight))
    a.train()
    with pytest.warns(UserWarning):
        a(torch.zeros_like(x))                            # zero mean: fallback direction, not frozen
    assert not a._v_ready_host
    a(x)
    assert a._v_ready_host and bool(a.v_ready)
    b = va.VeLoRALinear(128, 64, 32, device="cuda", dtype=torch.bfloat16)
    assert not b._v_ready_host
    b.load_state_dict(a.state_dict())
    assert b._v_ready_host and torch.equal(b.v, a.v)
    v0 = b.v.clone()
    b(x * 2.0)
    assert torch.equal(b.v, v0)                           # loaded v stays frozen
