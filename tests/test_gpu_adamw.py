"""GPU parity of the fused AdamW step on the factored gradient against the fp64 oracle."""
import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_helpers import rel_fro, to_dev

pytestmark = pytest.mark.gpu

# The boundary takes the hyper-parameters as C floats: both sides get the float32-representable values.
HYP = {k: float(np.float32(x)) for k, x in dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=1e-2).items()}

# float32 arithmetic against float64: the moments carry a few roundings each (relative 1e-6 is
# generous); the weight moves by about lr per step, so comparing the *movement* W_new - W_old
# adds the rounding of W itself, ulp(|W|)/2 ~ 3e-8*|W| against a movement of ~lr*|m/sqrt(u)|.
TOL_MOMENT = 2e-6
TOL_STEP_F32 = 2e-4      # |W| ~ 0.05, movement ~ 1e-3: 3e-8*0.05/1e-3 ~ 1.5e-6 per element, plus the division and sqrt


@pytest.fixture(scope="module")
def vl():
    import paper_2405_17991_amd as m
    return m


def _inputs(O, M, d, seed, w_bf16):
    D = M * d
    T = wl.random_tensor(O, M, wl.F32, seed, 11, 0.02)
    v = wl.random_unit_v(d, seed)
    W = wl.random_tensor(O, D, wl.BF16 if w_bf16 else wl.F32, seed, 12, 0.05)
    m = wl.random_tensor(O, D, wl.F32, seed, 13, 1e-3)
    u = np.square(wl.random_tensor(O, D, wl.F32, seed, 14, 1e-3)).astype(np.float32)
    return T, v, W, m, u


def _widen(W, w_bf16):
    return wl.bf16_bits_to_f32(W).astype(np.float64) if w_bf16 else W.astype(np.float64)


def _run(vl, T, v, W, m, u, w_bf16, step, grad_scale, zero_state=False):
    import torch
    if zero_state:
        m = np.zeros_like(m); u = np.zeros_like(u)
    Td, vd, md, ud = (torch.from_numpy(a.copy()).cuda() for a in (T, v, m, u))
    Wd = to_dev(W, wl.BF16 if w_bf16 else wl.F32)
    vl.velora_adamw_step_factor(Td, vd, Wd, md, ud, step=step, grad_scale=grad_scale, **HYP)
    torch.cuda.synchronize()
    W1 = Wd.view(torch.int16).cpu().numpy().view(np.uint16) if w_bf16 else Wd.cpu().numpy()
    eW, em, eu = oracle.adamw_step_factor(T, v, _widen(W, w_bf16), m, u, step=step, grad_scale=grad_scale, **HYP)
    return W1, md.cpu().numpy(), ud.cpu().numpy(), eW, em, eu


@pytest.mark.parametrize("O,M,d", [(64, 4, 16), (257, 43, 256), (33, 7, 12), (5, 3, 5), (130, 1, 64), (1, 1, 4)])
@pytest.mark.parametrize("step,zero_state", [(1, True), (7, False)])
def test_f32_weights(vl, O, M, d, step, zero_state):
    T, v, W, m, u = _inputs(O, M, d, 100 + O, False)
    W1, m1, u1, eW, em, eu = _run(vl, T, v, W, m, u, False, step, 0.5, zero_state)
    assert rel_fro(m1, em) <= TOL_MOMENT
    assert rel_fro(u1, eu) <= TOL_MOMENT
    W0 = W.astype(np.float64)
    assert rel_fro(W1.astype(np.float64) - W0, eW - W0) <= TOL_STEP_F32
    assert np.abs(W1 - eW).max() <= 4e-8 * max(1.0, np.abs(W0).max()) + 1e-3 * TOL_STEP_F32


@pytest.mark.parametrize("O,M,d", [(64, 4, 16), (257, 43, 256), (33, 7, 12), (5, 3, 5)])
def test_bf16_weights_round_once_on_store(vl, O, M, d):
    T, v, W, m, u = _inputs(O, M, d, 200 + O, True)
    W1, m1, u1, eW, em, eu = _run(vl, T, v, W, m, u, True, 3, 1.0)
    assert rel_fro(m1, em) <= TOL_MOMENT and rel_fro(u1, eu) <= TOL_MOMENT
    # the stored weight is the bf16 nearest to the updated value: compare bit patterns with the
    # oracle's value rounded the same way; a float32-vs-float64 difference next to a rounding
    # boundary may flip the last bit of a few elements
    exp_bits = wl.f32_to_bf16_bits(eW.astype(np.float32))
    diff = np.abs(W1.astype(np.int32) - exp_bits.astype(np.int32))
    assert diff.max() <= 1
    assert (diff != 0).mean() <= 0.01


def test_matches_expand_then_library_adamw_on_device(vl):
    # the same step taken the long way on the GPU: materialise dW with velora_expand_factor and
    # hand it to torch.optim.AdamW; the fused call must land on the same weights to rounding
    import torch
    O, M, d = 96, 6, 32
    T, v, W, m, u = _inputs(O, M, d, 7, False)
    Td, vd = torch.from_numpy(T).cuda(), torch.from_numpy(v).cuda()
    Wa = torch.from_numpy(W.copy()).cuda()
    ma, ua = torch.zeros_like(Wa), torch.zeros_like(Wa)
    p = torch.nn.Parameter(torch.from_numpy(W.copy()).cuda())
    opt = torch.optim.AdamW([p], lr=HYP["lr"], betas=(HYP["beta1"], HYP["beta2"]), eps=HYP["eps"],
                            weight_decay=HYP["weight_decay"])
    for step in range(1, 5):
        Ts = Td * float(step)
        vl.velora_adamw_step_factor(Ts, vd, Wa, ma, ua, step=step, **HYP)
        p.grad = vl.velora_expand_factor(Ts, vd, M * d)
        opt.step()
    torch.cuda.synchronize()
    W0 = torch.from_numpy(W).cuda()
    num = (Wa - p.detach()).double().norm().item()
    den = (p.detach() - W0).double().norm().item()
    assert num / den <= 1e-4


def test_full_size_llama7b_down_projection(vl):
    sh = wl.shape_by_name("cfg4_down")
    T, v, W, m, u = _inputs(sh.O, sh.M, sh.d, 31, False)
    W1, m1, u1, eW, em, eu = _run(vl, T, v, W, m, u, False, 5, 1.0)
    assert rel_fro(m1, em) <= TOL_MOMENT and rel_fro(u1, eu) <= TOL_MOMENT
    W0 = W.astype(np.float64)
    assert rel_fro(W1.astype(np.float64) - W0, eW - W0) <= TOL_STEP_F32


def test_rejects_bad_hyperparameters(vl):
    import torch
    T = torch.zeros(4, 2, device="cuda"); v = torch.ones(8, device="cuda")
    W = torch.zeros(4, 16, device="cuda"); m = torch.zeros_like(W); u = torch.zeros_like(W)
    with pytest.raises(vl.VeloraError):
        vl.velora_adamw_step_factor(T, v, W, m, u, lr=1e-3, step=0)
    with pytest.raises(vl.VeloraError):
        vl.velora_adamw_step_factor(T, v, W, m, u, lr=1e-3, beta1=1.0, step=1)
    assert not W.any()
