"""ctypes binding of libvelora (see include/velora.h for the contract).

Argument marshalling only.  Tensors are torch tensors on the GPU (PyTorch is
used for device memory and streams, nothing else); each wrapper checks dtype,
device and contiguity, then passes raw device pointers and sizes to the C ABI
on torch's current HIP stream.  ``M`` is the number of sub-tokens per token.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libvelora.so")

F32 = 0
BF16 = 1
OP_INIT_V = 0
OP_COMPRESS = 1
OP_RECONSTRUCT = 2
OP_WEIGHT_GRAD = 3
OP_WEIGHT_GRAD_FACTOR = 4

STATUS = {
    0: "VELORA_OK", 1: "VELORA_ERR_NULL", 2: "VELORA_ERR_SHAPE", 3: "VELORA_ERR_DTYPE",
    4: "VELORA_ERR_ALIGN", 5: "VELORA_ERR_WORKSPACE", 6: "VELORA_ERR_DEGENERATE", 7: "VELORA_ERR_HIP",
}

EXPORTS = [
    "velora_status_string", "velora_version", "velora_workspace_bytes", "velora_init_v",
    "velora_compress", "velora_reconstruct", "velora_weight_grad", "velora_weight_grad_static",
    "velora_weight_grad_factor",
    "velora_expand_factor", "velora_update_v", "velora_compress_update", "velora_adamw_step_factor",
    "velora_swiglu_compress", "velora_rmsnorm_compress", "velora_linear_compress", "velora_grad_input",
    "velora_bandwidth_probe",
]


class VeloraError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {velora_status_string(status)}")


def lib_path() -> str:
    return _LIB_PATH


def _load() -> ctypes.CDLL:
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build the HIP library first "
            "(python -m paper_2405_17991_amd.build, or __graft_entry__.build()). "
            "There is no fallback path.")
    L = ctypes.CDLL(_LIB_PATH)
    i64, vp, ci, sz = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    L.velora_status_string.argtypes = [ci]
    L.velora_status_string.restype = ctypes.c_char_p
    L.velora_version.argtypes = []
    L.velora_version.restype = ci
    L.velora_workspace_bytes.argtypes = [ci, i64, i64, i64, i64, ci]
    L.velora_workspace_bytes.restype = sz
    L.velora_init_v.argtypes = [vp, i64, i64, i64, ci, vp, vp, sz, vp]
    L.velora_init_v.restype = ci
    L.velora_compress.argtypes = [vp, vp, i64, i64, i64, ci, vp, vp]
    L.velora_compress.restype = ci
    L.velora_reconstruct.argtypes = [vp, vp, i64, i64, i64, ci, vp, vp]
    L.velora_reconstruct.restype = ci
    L.velora_weight_grad.argtypes = [vp, vp, vp, i64, i64, i64, i64, ci, vp, ci, ci, vp, sz, vp]
    L.velora_weight_grad.restype = ci
    L.velora_weight_grad_static.argtypes = [vp, vp, vp, i64, i64, i64, i64, ci, vp, ci, ci, vp]
    L.velora_weight_grad_static.restype = ci
    L.velora_weight_grad_factor.argtypes = [vp, vp, i64, i64, i64, ci, vp, vp, sz, vp]
    L.velora_weight_grad_factor.restype = ci
    L.velora_expand_factor.argtypes = [vp, vp, i64, i64, i64, vp, ci, ci, vp]
    L.velora_expand_factor.restype = ci
    L.velora_swiglu_compress.argtypes = [vp, vp, vp, i64, i64, i64, ci, vp, vp, vp]
    L.velora_swiglu_compress.restype = ci
    L.velora_linear_compress.argtypes = [vp, vp, vp, i64, i64, i64, i64, ci, vp, vp, vp]
    L.velora_linear_compress.restype = ci
    L.velora_grad_input.argtypes = [vp, vp, i64, i64, i64, ci, vp, vp]
    L.velora_grad_input.restype = ci
    L.velora_rmsnorm_compress.argtypes = [vp, vp, ctypes.c_float, vp, i64, i64, i64, ci, vp, vp, vp]
    L.velora_rmsnorm_compress.restype = ci
    cf = ctypes.c_float
    L.velora_adamw_step_factor.argtypes = [vp, vp, i64, i64, i64, vp, ci, vp, vp, cf, cf, cf, cf, cf, i64, cf, vp]
    L.velora_adamw_step_factor.restype = ci
    L.velora_bandwidth_probe.argtypes = [ci, vp, vp, i64, vp, vp]
    L.velora_bandwidth_probe.restype = ci
    L.velora_update_v.argtypes = [vp, i64, i64, i64, ci, vp, cf, vp, vp, sz, vp]
    L.velora_update_v.restype = ci
    L.velora_compress_update.argtypes = [vp, vp, i64, i64, i64, ci, vp, vp, cf, vp, vp, sz, vp]
    L.velora_compress_update.restype = ci
    return L


raw = _load()   # the C ABI itself, for callers that hold raw pointers


def velora_status_string(status: int) -> str:
    return raw.velora_status_string(int(status)).decode()


def velora_version() -> int:
    return int(raw.velora_version())


_ws_cache = {}
_torch_mod = None


def velora_workspace_bytes(op: int, N: int, D: int, O: int, M: int, dtype: int) -> int:
    # the answer depends on the current device's CU count, so the device is part of the key
    tm = _torch_mod
    dev = tm.cuda.current_device() if tm is not None and tm.cuda.is_initialized() else -1
    key = (dev, op, N, D, O, M, dtype)
    need = _ws_cache.get(key)
    if need is None:
        need = int(raw.velora_workspace_bytes(op, N, D, O, M, dtype))
        if len(_ws_cache) < 4096:
            _ws_cache[key] = need
    return need


# ---- torch plumbing ---------------------------------------------------------
def _torch():
    global _torch_mod
    if _torch_mod is None:
        import torch
        _torch_mod = torch
    return _torch_mod


def _dt(t) -> int:
    torch = _torch()
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}: expected float32 or bfloat16")


def _check(t, name: str, ndim: int):
    if not t.is_cuda:
        raise ValueError(f"{name} must be a GPU tensor")
    if t.dim() != ndim:
        raise ValueError(f"{name} must have {ndim} dimensions, got {tuple(t.shape)}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")


def _stream() -> int:
    return int(_torch().cuda.current_stream().cuda_stream)


def _ws(nbytes: int, like, ws):
    torch = _torch()
    if ws is None:
        ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=like.device)
    return ws


def _raise(st: int, where: str):
    if st != 0:
        raise VeloraError(st, where)


def velora_init_v(X, M: int, v=None, ws=None, allow_degenerate: bool = False):
    """v[d] = normalised mean of the N*M sub-tokens of X[N, D] (float32)."""
    torch = _torch()
    _check(X, "X", 2)
    N, D = X.shape
    if v is None:
        v = torch.empty(D // M if M > 0 and D % M == 0 else 1, dtype=torch.float32, device=X.device)
    _check(v, "v", 1)
    need = velora_workspace_bytes(OP_INIT_V, N, D, 0, M, _dt(X))
    ws = _ws(need, X, ws)
    st = raw.velora_init_v(X.data_ptr(), N, D, M, _dt(X), v.data_ptr(), ws.data_ptr(), ws.numel(), _stream())
    if st == 6 and allow_degenerate:
        return v
    _raise(st, "velora_init_v")
    return v


def velora_compress(X, v, M: int, S=None):
    """S[N, M] = <sub-token, v>, dtype of X."""
    torch = _torch()
    _check(X, "X", 2)
    _check(v, "v", 1)
    N, D = X.shape
    if v.dtype != torch.float32:
        raise TypeError("v must be float32")
    if M > 0 and D % M == 0 and v.numel() != D // M:
        raise ValueError(f"v must have D/M = {D // M} elements, got {v.numel()}")
    if S is None:
        S = torch.empty((N, max(M, 1)), dtype=X.dtype, device=X.device)
    _check(S, "S", 2)
    if S.dtype != X.dtype:
        raise TypeError("S must have X's dtype")
    st = raw.velora_compress(X.data_ptr(), v.data_ptr(), N, D, M, _dt(X), S.data_ptr(), _stream())
    _raise(st, "velora_compress")
    return S


def velora_swiglu_compress(gate, up, v, M: int, X=None, S=None):
    """X = silu(gate) * up and S = compress(X, v) in one pass.  -> (X, S)"""
    torch = _torch()
    _check(gate, "gate", 2)
    _check(up, "up", 2)
    _check(v, "v", 1)
    if gate.shape != up.shape or gate.dtype != up.dtype:
        raise ValueError("gate and up must have the same shape and dtype")
    if v.dtype != torch.float32:
        raise TypeError("v must be float32")
    N, D = gate.shape
    if X is None:
        X = torch.empty_like(gate)
    if S is None:
        S = torch.empty((N, max(M, 1)), dtype=gate.dtype, device=gate.device)
    _check(X, "X", 2)
    _check(S, "S", 2)
    if tuple(X.shape) != (N, D) or X.dtype != gate.dtype or tuple(S.shape) != (N, M) or S.dtype != gate.dtype:
        raise ValueError("X must be [N, D] and S [N, M] in the inputs' dtype")
    st = raw.velora_swiglu_compress(gate.data_ptr(), up.data_ptr(), v.data_ptr(), N, D, M, _dt(gate), X.data_ptr(),
                                    S.data_ptr(), _stream())
    _raise(st, "velora_swiglu_compress")
    return X, S


def velora_linear_compress(X, W, v, M: int, Y=None, S=None):
    """Y = X @ W^T (W is [O, D]) and S = compress(X, v) from one pass over X.  -> (Y, S)"""
    torch = _torch()
    _check(X, "X", 2)
    _check(W, "W", 2)
    _check(v, "v", 1)
    if W.dtype != X.dtype or W.shape[1] != X.shape[1]:
        raise ValueError("W must be [O, D] in X's dtype")
    if v.dtype != torch.float32:
        raise TypeError("v must be float32")
    N, D = X.shape
    O = W.shape[0]
    if Y is None:
        Y = torch.empty((N, O), dtype=X.dtype, device=X.device)
    if S is None:
        S = torch.empty((N, max(M, 1)), dtype=X.dtype, device=X.device)
    _check(Y, "Y", 2)
    _check(S, "S", 2)
    if tuple(Y.shape) != (N, O) or Y.dtype != X.dtype or tuple(S.shape) != (N, M) or S.dtype != X.dtype:
        raise ValueError("Y must be [N, O] and S [N, M] in X's dtype")
    st = raw.velora_linear_compress(X.data_ptr(), W.data_ptr(), v.data_ptr(), N, D, O, M, _dt(X), Y.data_ptr(),
                                    S.data_ptr(), _stream())
    _raise(st, "velora_linear_compress")
    return Y, S


def velora_grad_input(G, W, dX=None):
    """dX = G @ W (G is [N, O], W is [O, D]): the input gradient of the layer.  -> dX [N, D]"""
    torch = _torch()
    _check(G, "G", 2)
    _check(W, "W", 2)
    if W.dtype != G.dtype or W.shape[0] != G.shape[1]:
        raise ValueError("W must be [O, D] in G's dtype")
    N, O = G.shape
    D = W.shape[1]
    if dX is None:
        dX = torch.empty((N, D), dtype=G.dtype, device=G.device)
    _check(dX, "dX", 2)
    if tuple(dX.shape) != (N, D) or dX.dtype != G.dtype:
        raise ValueError("dX must be [N, D] in G's dtype")
    st = raw.velora_grad_input(G.data_ptr(), W.data_ptr(), N, O, D, _dt(G), dX.data_ptr(), _stream())
    _raise(st, "velora_grad_input")
    return dX


def velora_rmsnorm_compress(H, gamma, eps: float, v, M: int, X=None, S=None):
    """X = RMSNorm(H) * gamma and S = compress(X, v) in one pass.  -> (X, S)"""
    torch = _torch()
    _check(H, "H", 2)
    _check(gamma, "gamma", 1)
    _check(v, "v", 1)
    if v.dtype != torch.float32 or gamma.dtype != torch.float32:
        raise TypeError("gamma and v must be float32")
    N, D = H.shape
    if gamma.numel() != D:
        raise ValueError("gamma must be [D]")
    if X is None:
        X = torch.empty_like(H)
    if S is None:
        S = torch.empty((N, max(M, 1)), dtype=H.dtype, device=H.device)
    _check(X, "X", 2)
    _check(S, "S", 2)
    if tuple(X.shape) != (N, D) or X.dtype != H.dtype or tuple(S.shape) != (N, M) or S.dtype != H.dtype:
        raise ValueError("X must be [N, D] and S [N, M] in H's dtype")
    st = raw.velora_rmsnorm_compress(H.data_ptr(), gamma.data_ptr(), float(eps), v.data_ptr(), N, D, M, _dt(H),
                                     X.data_ptr(), S.data_ptr(), _stream())
    _raise(st, "velora_rmsnorm_compress")
    return X, S


def velora_reconstruct(S, v, D: int, Xhat=None):
    """Xhat[N, D] with Xhat[n, g*d + j] = S[n, g] * v[j], dtype of S."""
    torch = _torch()
    _check(S, "S", 2)
    _check(v, "v", 1)
    N, M = S.shape
    if v.dtype != torch.float32:
        raise TypeError("v must be float32")
    if Xhat is None:
        Xhat = torch.empty((N, D), dtype=S.dtype, device=S.device)
    _check(Xhat, "Xhat", 2)
    st = raw.velora_reconstruct(S.data_ptr(), v.data_ptr(), N, D, M, _dt(S), Xhat.data_ptr(), _stream())
    _raise(st, "velora_reconstruct")
    return Xhat


def velora_weight_grad(G, S, v, D: int, dW=None, dw_dtype=None, accumulate: bool = False, ws=None):
    """dW[O, D] (+)= G^T @ ungroup(reconstruct(S, v)) without forming Xhat."""
    torch = _torch()
    _check(G, "G", 2)
    _check(S, "S", 2)
    _check(v, "v", 1)
    N, O = G.shape
    N2, M = S.shape
    if N2 != N:
        raise ValueError("G and S must have the same number of tokens")
    if G.dtype != S.dtype:
        raise TypeError("G and S must share a dtype")
    if v.dtype != torch.float32:
        raise TypeError("v must be float32")
    if dW is None:
        if accumulate:
            raise ValueError("accumulate=True needs an existing dW")
        dW = torch.empty((O, D), dtype=dw_dtype or torch.float32, device=G.device)
    _check(dW, "dW", 2)
    if tuple(dW.shape) != (O, D):
        raise ValueError(f"dW must be [{O}, {D}]")
    need = velora_workspace_bytes(OP_WEIGHT_GRAD, N, D, O, M, _dt(G))
    ws = _ws(need, G, ws)
    st = raw.velora_weight_grad(G.data_ptr(), S.data_ptr(), v.data_ptr(), N, O, D, M, _dt(G), dW.data_ptr(),
                                _dt(dW), 1 if accumulate else 0, ws.data_ptr(), ws.numel(), _stream())
    _raise(st, "velora_weight_grad")
    return dW


def velora_weight_grad_static(G, S, v, D: int, dW, accumulate: bool = False):
    """velora_weight_grad on the library's static device scratch: no workspace argument and no allocation
    anywhere (the caller passes dW).  Shapes that need more than VELORA_STATIC_SCRATCH_BYTES raise
    VELORA_ERR_WORKSPACE; calls that may overlap on one GPU must be serialised by the caller."""
    torch = _torch()
    _check(G, "G", 2)
    _check(S, "S", 2)
    _check(v, "v", 1)
    _check(dW, "dW", 2)
    N, O = G.shape
    N2, M = S.shape
    if N2 != N:
        raise ValueError("G and S must have the same number of tokens")
    if G.dtype != S.dtype:
        raise TypeError("G and S must share a dtype")
    if v.dtype != torch.float32:
        raise TypeError("v must be float32")
    if tuple(dW.shape) != (O, D):
        raise ValueError(f"dW must be [{O}, {D}]")
    st = raw.velora_weight_grad_static(G.data_ptr(), S.data_ptr(), v.data_ptr(), N, O, D, M, _dt(G), dW.data_ptr(),
                                       _dt(dW), 1 if accumulate else 0, _stream())
    _raise(st, "velora_weight_grad_static")
    return dW


def velora_bandwidth_probe(kind: str, src=None, dst=None, sink=None):
    """The library's plainest streaming kernels (a measurement aid): kind 'read' (src, sink = 64 int32),
    'write' (dst) or 'copy' (src -> dst), over the whole tensors."""
    k = {"read": 0, "write": 1, "copy": 2}[kind]
    t = src if k != 1 else dst
    nbytes = t.numel() * t.element_size()
    st = raw.velora_bandwidth_probe(k, src.data_ptr() if src is not None else None,
                                    dst.data_ptr() if dst is not None else None, nbytes,
                                    sink.data_ptr() if sink is not None else None, _stream())
    _raise(st, "velora_bandwidth_probe")


STATIC_SCRATCH_BYTES = 64 << 20     # VELORA_STATIC_SCRATCH_BYTES of include/velora.h


def velora_weight_grad_factor(G, S, T=None, ws=None):
    """T[O, M] = G^T S (float32): the factor of the weight gradient, d times smaller than dW."""
    torch = _torch()
    _check(G, "G", 2)
    _check(S, "S", 2)
    N, O = G.shape
    N2, M = S.shape
    if N2 != N:
        raise ValueError("G and S must have the same number of tokens")
    if G.dtype != S.dtype:
        raise TypeError("G and S must share a dtype")
    if T is None:
        T = torch.empty((O, M), dtype=torch.float32, device=G.device)
    _check(T, "T", 2)
    if tuple(T.shape) != (O, M) or T.dtype != torch.float32:
        raise ValueError(f"T must be float32 [{O}, {M}]")
    need = velora_workspace_bytes(OP_WEIGHT_GRAD_FACTOR, N, M, O, M, _dt(G))
    ws = _ws(need, G, ws)
    st = raw.velora_weight_grad_factor(G.data_ptr(), S.data_ptr(), N, O, M, _dt(G), T.data_ptr(), ws.data_ptr(),
                                       ws.numel(), _stream())
    _raise(st, "velora_weight_grad_factor")
    return T


def velora_expand_factor(T, v, D: int, dW=None, dw_dtype=None, accumulate: bool = False):
    """dW[o, g*d + j] (+)= T[o, g] * v[j]."""
    torch = _torch()
    _check(T, "T", 2)
    _check(v, "v", 1)
    O, M = T.shape
    if T.dtype != torch.float32 or v.dtype != torch.float32:
        raise TypeError("T and v must be float32")
    if dW is None:
        if accumulate:
            raise ValueError("accumulate=True needs an existing dW")
        dW = torch.empty((O, D), dtype=dw_dtype or torch.float32, device=T.device)
    _check(dW, "dW", 2)
    if tuple(dW.shape) != (O, D):
        raise ValueError(f"dW must be [{O}, {D}]")
    st = raw.velora_expand_factor(T.data_ptr(), v.data_ptr(), O, D, M, dW.data_ptr(), _dt(dW),
                                  1 if accumulate else 0, _stream())
    _raise(st, "velora_expand_factor")
    return dW


def velora_adamw_step_factor(T, v, W, exp_avg, exp_avg_sq, *, lr: float, beta1: float = 0.9, beta2: float = 0.999,
                             eps: float = 1e-8, weight_decay: float = 1e-2, step: int, grad_scale: float = 1.0):
    """One in-place AdamW step on W[O, D] from the factored gradient grad_scale * T (x) v."""
    torch = _torch()
    _check(T, "T", 2)
    _check(v, "v", 1)
    _check(W, "W", 2)
    _check(exp_avg, "exp_avg", 2)
    _check(exp_avg_sq, "exp_avg_sq", 2)
    O, M = T.shape
    D = W.shape[1]
    if T.dtype != torch.float32 or v.dtype != torch.float32:
        raise TypeError("T and v must be float32")
    if exp_avg.dtype != torch.float32 or exp_avg_sq.dtype != torch.float32:
        raise TypeError("exp_avg and exp_avg_sq must be float32")
    if W.shape[0] != O or tuple(exp_avg.shape) != tuple(W.shape) or tuple(exp_avg_sq.shape) != tuple(W.shape):
        raise ValueError(f"W, exp_avg and exp_avg_sq must be [{O}, D]")
    if M <= 0 or D % M or v.numel() != D // M:
        raise ValueError("v must be [D / M]")
    st = raw.velora_adamw_step_factor(T.data_ptr(), v.data_ptr(), O, D, M, W.data_ptr(), _dt(W), exp_avg.data_ptr(),
                                      exp_avg_sq.data_ptr(), float(lr), float(beta1), float(beta2), float(eps),
                                      float(weight_decay), int(step), float(grad_scale), _stream())
    _raise(st, "velora_adamw_step_factor")
    return W


def velora_update_v(X, M: int, mean_state=None, beta: float = 0.0, v=None, ws=None):
    """Per-batch vector: v = normalise(beta * mean_state + (1 - beta) * batch mean); asynchronous."""
    torch = _torch()
    _check(X, "X", 2)
    N, D = X.shape
    d = D // M if M > 0 and D % M == 0 else 1
    if v is None:
        v = torch.empty(d, dtype=torch.float32, device=X.device)
    _check(v, "v", 1)
    if mean_state is not None:
        _check(mean_state, "mean_state", 1)
        if mean_state.dtype != torch.float32 or mean_state.numel() != d:
            raise ValueError("mean_state must be float32 [d]")
    need = velora_workspace_bytes(OP_INIT_V, N, D, 0, M, _dt(X))
    ws = _ws(need, X, ws)
    st = raw.velora_update_v(X.data_ptr(), N, D, M, _dt(X), None if mean_state is None else mean_state.data_ptr(),
                             float(beta), v.data_ptr(), ws.data_ptr(), ws.numel(), _stream())
    _raise(st, "velora_update_v")
    return v


def velora_compress_update(X, v_in, M: int, mean_state=None, beta: float = 0.0, S=None, v_out=None, ws=None):
    """One pass: S = compress(X, v_in) and (mean_state, v_out) updated from X.  -> (S, v_out)"""
    torch = _torch()
    _check(X, "X", 2)
    _check(v_in, "v_in", 1)
    N, D = X.shape
    if v_in.dtype != torch.float32:
        raise TypeError("v_in must be float32")
    if S is None:
        S = torch.empty((N, max(M, 1)), dtype=X.dtype, device=X.device)
    _check(S, "S", 2)
    if v_out is None:
        v_out = torch.empty_like(v_in)
    _check(v_out, "v_out", 1)
    if mean_state is not None:
        _check(mean_state, "mean_state", 1)
    need = velora_workspace_bytes(OP_INIT_V, N, D, 0, M, _dt(X))
    ws = _ws(need, X, ws)
    st = raw.velora_compress_update(X.data_ptr(), v_in.data_ptr(), N, D, M, _dt(X), S.data_ptr(),
                                    None if mean_state is None else mean_state.data_ptr(), float(beta),
                                    v_out.data_ptr(), ws.data_ptr(), ws.numel(), _stream())
    _raise(st, "velora_compress_update")
    return S, v_out
