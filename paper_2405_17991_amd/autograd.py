"""A linear layer that trains with VeLoRA's compressed activations (paper
Algorithm 1), wired into PyTorch autograd.

Forward: the dense product is untouched (``out = input @ weight.T`` through the
vendor GEMM, "forward compute is preserved"); next to it the library's compress
kernel produces ``S[N, M]`` and *that* is what autograd keeps instead of the
input.  Backward: ``grad_input = grad_output @ weight`` (vendor GEMM, does not
need the input) and ``grad_weight`` from ``velora_weight_grad`` on
``(grad_output, S, v)``; the reconstructed input is never formed.  ``v`` is set
from the first batch (Sec. 3.3) and then frozen.

Only the two VeLoRA steps run in this package's kernels; the two dense GEMMs
are not part of the method and use ``torch.matmul``.  The saved activation
shrinks from ``N*D`` to ``N*M = N*D/d`` elements (Sec. 3.2).
"""
from __future__ import annotations

from typing import Optional

import torch

from . import binding as _b


class VeLoRALinearFunction(torch.autograd.Function):
    """``forward(input[..., D], weight[O, D], v[d], M) -> out[..., O]``."""

    @staticmethod
    def forward(ctx, input, weight, v, M):
        D = input.shape[-1]
        x2 = input.reshape(-1, D)
        if not x2.is_contiguous():
            x2 = x2.contiguous()
        out = torch.matmul(x2, weight.t())
        S = _b.velora_compress(x2, v, M)          # the only activation kept for backward
        ctx.save_for_backward(S, weight, v)
        ctx.in_shape = input.shape
        ctx.needs_in = ctx.needs_input_grad[0]
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
            grad_input = torch.matmul(g2, weight).reshape(ctx.in_shape)
        grad_weight = None
        if ctx.needs_input_grad[1]:
            grad_weight = _b.velora_weight_grad(g2, S, v, D, dw_dtype=weight.dtype)
        return grad_input, grad_weight, None, None


class VeLoRALinear(torch.nn.Module):
    """Bias-free linear layer whose backward uses rank-1 sub-token projections.

    ``sub_token_size`` is d (the paper's "M"); ``in_features`` must be a
    multiple of it.  ``v`` is a buffer: initialised from the first batch seen in
    training mode, then fixed and saved with the module's state.
    """

    def __init__(self, in_features: int, out_features: int, sub_token_size: int, device=None, dtype=None):
        super().__init__()
        if in_features % sub_token_size:
            raise ValueError("sub_token_size must divide in_features")
        self.in_features, self.out_features, self.d = in_features, out_features, sub_token_size
        self.M = in_features // sub_token_size
        w = torch.empty((out_features, in_features), device=device, dtype=dtype)
        torch.nn.init.normal_(w, std=in_features ** -0.5)
        self.weight = torch.nn.Parameter(w)
        self.register_buffer("v", torch.zeros(sub_token_size, device=device, dtype=torch.float32))
        self.register_buffer("v_ready", torch.zeros((), device=device, dtype=torch.bool))

    @torch.no_grad()
    def init_v(self, batch: torch.Tensor) -> None:
        x2 = batch.reshape(-1, self.in_features).contiguous()
        _b.velora_init_v(x2, self.M, v=self.v, allow_degenerate=True)
        self.v_ready.fill_(True)

    def forward(self, input: torch.Tensor) -> torch.Tensor:
        if not bool(self.v_ready):
            self.init_v(input.detach())
        return VeLoRALinearFunction.apply(input, self.weight, self.v, self.M)


def saved_activation_bytes(N: int, D: int, d: int, elem_bytes: int = 2) -> dict:
    """Closed form behind the paper's activation-memory tables: what one layer
    keeps for backward with and without VeLoRA (ratio = d)."""
    return {"baseline": N * D * elem_bytes, "velora": N * (D // d) * elem_bytes, "ratio": float(d)}
