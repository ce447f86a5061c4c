"""A linear layer that trains with VeLoRA's compressed activations (paper
Listing 1), wired into PyTorch autograd.

Forward: the dense product is untouched (``out = input @ weight.T`` through the
vendor GEMM: the listing leaves the dense product as it is); next to it the library's compress
kernel produces ``S[N, M]`` and *that* is what autograd keeps instead of the
input.  Backward: ``grad_input = grad_output @ weight`` (vendor GEMM, does not
need the input) and ``grad_weight`` from ``velora_weight_grad`` on
``(grad_output, S, v)``; the reconstructed input is never formed.  ``v`` is set
from the first batch (Sec. 3.2) and then frozen.

Only the two VeLoRA steps run in this package's kernels; the two dense GEMMs
are not part of the method and use ``torch.matmul``.  The saved activation
shrinks from ``N*D`` to ``N*M = N*D/d`` elements (Sec. 3.1).

``VeLoRALlamaMLP`` applies the same rule to a whole gated MLP block: the block
input is compressed once for the gate and up projections, and the down
projection's input is compressed by the kernel that produces it.
``VeLoRANormLinears`` does it for the input side of an attention block: RMSNorm
and compress in one kernel, one S for the q, k and v projections.
"""
from __future__ import annotations

import warnings
from typing import Optional

import torch

from . import binding as _b


class _FirstBatchV(torch.nn.Module):
    """What the three wrapper modules share: the "is v set" flag.

    ``v_ready`` is a buffer so that it travels with the state dict, but reading a device buffer
    costs a device-to-host synchronisation; ``forward`` therefore looks at a host-side mirror
    that ``init_v`` and state-dict loading keep in step.  ``v`` is taken from the first batch
    seen in TRAINING mode (Sec. 3.2, "Cheap initialisation strategies"); a batch whose sub-token
    mean is zero or not finite leaves the library's fallback direction in ``v`` for that batch
    only, warns, and the next training batch tries again.
    """

    def _register_ready(self, device) -> None:
        self.register_buffer("v_ready", torch.zeros((), device=device, dtype=torch.bool))
        self._v_ready_host = False

    def _load_from_state_dict(self, state_dict, prefix, *args, **kwargs):
        super()._load_from_state_dict(state_dict, prefix, *args, **kwargs)
        key = prefix + "v_ready"
        if key in state_dict:
            self._v_ready_host = bool(state_dict[key])     # one read at load time, none per step

    def _init_vectors(self, pairs) -> None:
        """pairs: [(batch [n, D], M, v buffer)]; sets the flag only if every mean was usable."""
        ok = True
        for x2, M, v in pairs:
            try:
                _b.velora_init_v(x2, M, v=v)
            except _b.VeloraError as e:
                if e.status != 6:
                    raise
                ok = False
                warnings.warn("VeLoRA: the first batch's sub-token mean is zero or not finite; using the "
                              "uniform direction for this batch and initialising v again from the next one")
        if ok:
            self.v_ready.fill_(True)
            self._v_ready_host = True

    def _need_v(self) -> bool:
        """True when forward must initialise v first.  Outside training mode an uninitialised module
        runs the plain dense forward (exact gradients, nothing compressed) instead."""
        return self.training and not self._v_ready_host


class VeLoRALinearFunction(torch.autograd.Function):
    """``forward(input[..., D], weight[O, D], v[d], M, own_gemm=False) -> out[..., O]``.

    ``own_gemm``: run the two dense products in this package's kernels as well
    (``velora_linear_compress`` forms the output and S from one pass over the
    input; ``velora_grad_input`` the input gradient) instead of the vendor GEMM.
    """

    @staticmethod
    def forward(ctx, input, weight, v, M, own_gemm=False):
        D = input.shape[-1]
        x2 = input.reshape(-1, D)
        if not x2.is_contiguous():
            x2 = x2.contiguous()
        if own_gemm:
            out, S = _b.velora_linear_compress(x2, weight.detach().contiguous(), v, M)
        else:
            out = torch.matmul(x2, weight.t())
            S = _b.velora_compress(x2, v, M)      # the only activation kept for backward
        ctx.save_for_backward(S, weight, v)
        ctx.in_shape = input.shape
        ctx.needs_in = ctx.needs_input_grad[0]
        ctx.own_gemm = own_gemm
        return out.reshape(*input.shape[:-1], weight.shape[0])

    @staticmethod
    def backward(ctx, grad_output):
        S, weight, v = ctx.saved_tensors
        O, D = weight.shape
        g2 = grad_output.reshape(-1, O)
        if not g2.is_contiguous():
            g2 = g2.contiguous()
        grad_input = None
        if ctx.needs_in:
            if ctx.own_gemm:
                grad_input = _b.velora_grad_input(g2, weight.detach().contiguous()).reshape(ctx.in_shape)
            else:
                grad_input = torch.matmul(g2, weight).reshape(ctx.in_shape)
        grad_weight = None
        if ctx.needs_input_grad[1]:
            grad_weight = _b.velora_weight_grad(g2, S, v, D, dw_dtype=weight.dtype)
        return grad_input, grad_weight, None, None, None


class VeLoRALinear(_FirstBatchV):
    """Bias-free linear layer whose backward uses rank-1 sub-token projections.

    ``sub_token_size`` is d (the paper's "M"); ``in_features`` must be a
    multiple of it.  ``v`` is a buffer: initialised from the first batch seen in
    training mode, then fixed and saved with the module's state.
    """

    def __init__(self, in_features: int, out_features: int, sub_token_size: int, device=None, dtype=None,
                 own_gemm: bool = False):
        super().__init__()
        if in_features % sub_token_size:
            raise ValueError("sub_token_size must divide in_features")
        self.own_gemm = own_gemm
        self.in_features, self.out_features, self.d = in_features, out_features, sub_token_size
        self.M = in_features // sub_token_size
        w = torch.empty((out_features, in_features), device=device, dtype=dtype)
        torch.nn.init.normal_(w, std=in_features ** -0.5)
        self.weight = torch.nn.Parameter(w)
        self.register_buffer("v", torch.zeros(sub_token_size, device=device, dtype=torch.float32))
        self._register_ready(device)

    @torch.no_grad()
    def init_v(self, batch: torch.Tensor) -> None:
        self._init_vectors([(batch.reshape(-1, self.in_features).contiguous(), self.M, self.v)])

    def forward(self, input: torch.Tensor) -> torch.Tensor:
        if self._need_v():
            self.init_v(input.detach())
        elif not self._v_ready_host:        # evaluation before any training batch: the plain layer
            return torch.nn.functional.linear(input, self.weight)
        return VeLoRALinearFunction.apply(input, self.weight, self.v, self.M, self.own_gemm)


def saved_activation_bytes(N: int, D: int, d: int, elem_bytes: int = 2) -> dict:
    """Closed form behind the paper's activation-memory tables: what one layer
    keeps for backward with and without VeLoRA (ratio = d)."""
    return {"baseline": N * D * elem_bytes, "velora": N * (D // d) * elem_bytes, "ratio": float(d)}


class _SharedInputLinearsFunction(torch.autograd.Function):
    """Two bias-free linears on the same input (an MLP's gate and up projections):
    the input is compressed ONCE and both weight gradients are formed from the
    same S (Listing 1 applied to each layer; the saved tensor is shared)."""

    @staticmethod
    def forward(ctx, input, w_a, w_b, v, M):
        D = input.shape[-1]
        x2 = input.reshape(-1, D)
        if not x2.is_contiguous():
            x2 = x2.contiguous()
        S = _b.velora_compress(x2, v, M)
        out_a = torch.matmul(x2, w_a.t())
        out_b = torch.matmul(x2, w_b.t())
        ctx.save_for_backward(S, w_a, w_b, v)
        ctx.in_shape = input.shape
        lead = input.shape[:-1]
        return out_a.reshape(*lead, w_a.shape[0]), out_b.reshape(*lead, w_b.shape[0])

    @staticmethod
    def backward(ctx, g_a, g_b):
        S, w_a, w_b, v = ctx.saved_tensors
        D = w_a.shape[1]
        ga = g_a.reshape(-1, w_a.shape[0]).contiguous()
        gb = g_b.reshape(-1, w_b.shape[0]).contiguous()
        grad_input = None
        if ctx.needs_input_grad[0]:
            grad_input = (torch.matmul(ga, w_a) + torch.matmul(gb, w_b)).reshape(ctx.in_shape)
        dwa = _b.velora_weight_grad(ga, S, v, D, dw_dtype=w_a.dtype) if ctx.needs_input_grad[1] else None
        dwb = _b.velora_weight_grad(gb, S, v, D, dw_dtype=w_b.dtype) if ctx.needs_input_grad[2] else None
        return grad_input, dwa, dwb, None, None


class _SwiGLUDownFunction(torch.autograd.Function):
    """``out = (silu(gate) * up) @ weight.T`` with the product compressed where it is
    produced (``velora_swiglu_compress``): the product itself is not kept for
    backward, only S; gate and up stay because the activation's own backward
    needs them."""

    @staticmethod
    def forward(ctx, gate, up, weight, v, M):
        F = gate.shape[-1]
        g2 = gate.reshape(-1, F).contiguous()
        u2 = up.reshape(-1, F).contiguous()
        X, S = _b.velora_swiglu_compress(g2, u2, v, M)
        out = torch.matmul(X, weight.t())
        del X
        ctx.save_for_backward(g2, u2, S, weight, v)
        ctx.in_shape = gate.shape
        return out.reshape(*gate.shape[:-1], weight.shape[0])

    @staticmethod
    def backward(ctx, grad_output):
        g2, u2, S, weight, v = ctx.saved_tensors
        O, F = weight.shape
        go = grad_output.reshape(-1, O).contiguous()
        grad_w = _b.velora_weight_grad(go, S, v, F, dw_dtype=weight.dtype) if ctx.needs_input_grad[2] else None
        grad_gate = grad_up = None
        if ctx.needs_input_grad[0] or ctx.needs_input_grad[1]:
            dX = torch.matmul(go, weight).float()
            gf = g2.float()
            sig = torch.sigmoid(gf)
            grad_up = (dX * gf * sig).to(u2.dtype).reshape(ctx.in_shape)
            grad_gate = (dX * u2.float() * sig * (1.0 + gf * (1.0 - sig))).to(g2.dtype).reshape(ctx.in_shape)
        return grad_gate, grad_up, grad_w, None, None


class VeLoRALlamaMLP(_FirstBatchV):
    """LLaMA-style gated MLP, ``down(silu(gate(h)) * up(h))``, with VeLoRA on all three
    projections: ``h`` is compressed once for gate and up, and the down
    projection's input is compressed in the kernel that produces it.  Per token the
    block keeps ``hidden/d_h + inter/d_ff`` scalars in place of ``hidden + inter``
    saved inputs (gate and up themselves are still kept for the activation)."""

    def __init__(self, hidden: int, inter: int, d_hidden: int, d_inter: int, device=None, dtype=None):
        super().__init__()
        if hidden % d_hidden or inter % d_inter:
            raise ValueError("the sub-token sizes must divide the layer widths")
        self.hidden, self.inter = hidden, inter
        self.M_h, self.M_f = hidden // d_hidden, inter // d_inter
        mk = lambda o, i: torch.nn.Parameter(torch.nn.init.normal_(torch.empty((o, i), device=device, dtype=dtype),
                                                                    std=i ** -0.5))
        self.w_gate, self.w_up, self.w_down = mk(inter, hidden), mk(inter, hidden), mk(hidden, inter)
        self.register_buffer("v_h", torch.zeros(d_hidden, device=device, dtype=torch.float32))
        self.register_buffer("v_f", torch.zeros(d_inter, device=device, dtype=torch.float32))
        self._register_ready(device)

    @torch.no_grad()
    def init_v(self, h: torch.Tensor) -> None:
        """Both vectors from the first batch (Sec. 3.2): v_h from h, v_f from the first silu(gate)*up."""
        h2 = h.reshape(-1, self.hidden).contiguous()
        x = torch.nn.functional.silu(torch.matmul(h2, self.w_gate.t())) * torch.matmul(h2, self.w_up.t())
        self._init_vectors([(h2, self.M_h, self.v_h), (x.contiguous(), self.M_f, self.v_f)])

    def forward(self, h: torch.Tensor) -> torch.Tensor:
        if self._need_v():
            self.init_v(h.detach())
        elif not self._v_ready_host:
            F = torch.nn.functional
            return F.linear(F.silu(F.linear(h, self.w_gate)) * F.linear(h, self.w_up), self.w_down)
        gate, up = _SharedInputLinearsFunction.apply(h, self.w_gate, self.w_up, self.v_h, self.M_h)
        return _SwiGLUDownFunction.apply(gate, up, self.w_down, self.v_f, self.M_f)


class _NormLinearsFunction(torch.autograd.Function):
    """RMSNorm followed by several bias-free linears on the normalised input (an attention block's
    q, k, v projections; the paper's LLaMA runs compress the value projection's input, Sec. 4).
    ``velora_rmsnorm_compress`` writes the normalised input X and S = compress(X, v) in one pass;
    X feeds the dense products and is then dropped, S is kept once for all the weight gradients,
    and h stays because the normalisation's own backward needs it (as it does without VeLoRA)."""

    @staticmethod
    def forward(ctx, h, gamma, v, M, eps, *weights):
        H = h.shape[-1]
        h2 = h.reshape(-1, H)
        if not h2.is_contiguous():
            h2 = h2.contiguous()
        X, S = _b.velora_rmsnorm_compress(h2, gamma, eps, v, M)
        outs = tuple(torch.matmul(X, w.t()).reshape(*h.shape[:-1], w.shape[0]) for w in weights)
        del X
        ctx.save_for_backward(h2, gamma, S, v, *weights)
        ctx.in_shape, ctx.eps = h.shape, eps
        return outs

    @staticmethod
    def backward(ctx, *grads):
        h2, gamma, S, v, *weights = ctx.saved_tensors
        H = h2.shape[1]
        gs = [g.reshape(-1, w.shape[0]).contiguous() for g, w in zip(grads, weights)]
        grad_ws = [(_b.velora_weight_grad(g, S, v, H, dw_dtype=w.dtype) if ctx.needs_input_grad[5 + i] else None)
                   for i, (g, w) in enumerate(zip(gs, weights))]
        grad_h = grad_gamma = None
        if ctx.needs_input_grad[0] or ctx.needs_input_grad[1]:
            dX = torch.matmul(gs[0], weights[0]).float()
            for g, w in zip(gs[1:], weights[1:]):
                dX += torch.matmul(g, w).float()
            hf = h2.float()
            rinv = torch.rsqrt(hf.pow(2).mean(dim=-1, keepdim=True) + ctx.eps)
            xhat = hf * rinv
            if ctx.needs_input_grad[1]:
                grad_gamma = (dX * xhat).sum(dim=0)
            if ctx.needs_input_grad[0]:
                dxg = dX * gamma
                grad_h = (rinv * (dxg - xhat * (dxg * xhat).mean(dim=-1, keepdim=True))).to(h2.dtype).reshape(ctx.in_shape)
        return (grad_h, grad_gamma, None, None, None, *grad_ws)


class VeLoRANormLinears(_FirstBatchV):
    """``RMSNorm(h) -> [linear_i]``: the input side of a LLaMA attention block (q, k, v) with VeLoRA on the
    projections.  ``out_features`` lists the projections' widths; one ``v`` and one ``S`` serve all of them."""

    def __init__(self, hidden: int, out_features, sub_token_size: int, eps: float = 1e-5, device=None, dtype=None):
        super().__init__()
        if hidden % sub_token_size:
            raise ValueError("sub_token_size must divide the hidden width")
        self.hidden, self.M, self.eps = hidden, hidden // sub_token_size, eps
        self.gamma = torch.nn.Parameter(torch.ones(hidden, device=device, dtype=torch.float32))
        self.weights = torch.nn.ParameterList(
            [torch.nn.Parameter(torch.nn.init.normal_(torch.empty((o, hidden), device=device, dtype=dtype),
                                                      std=hidden ** -0.5)) for o in out_features])
        self.register_buffer("v", torch.zeros(sub_token_size, device=device, dtype=torch.float32))
        self._register_ready(device)

    def _normalised(self, h: torch.Tensor) -> torch.Tensor:
        hf = h.reshape(-1, self.hidden).float()
        return (hf * torch.rsqrt(hf.pow(2).mean(dim=-1, keepdim=True) + self.eps) * self.gamma).to(h.dtype)

    @torch.no_grad()
    def init_v(self, h: torch.Tensor) -> None:
        """v from the first batch's normalised input (Sec. 3.2, "Cheap initialisation strategies")."""
        self._init_vectors([(self._normalised(h).contiguous(), self.M, self.v)])

    def forward(self, h: torch.Tensor):
        if self._need_v():
            self.init_v(h.detach())
        elif not self._v_ready_host:
            x = self._normalised(h).reshape(h.shape)
            return tuple(torch.nn.functional.linear(x, w) for w in self.weights)
        return _NormLinearsFunction.apply(h, self.gamma, self.v, self.M, self.eps, *self.weights)
