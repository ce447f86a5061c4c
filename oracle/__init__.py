"""CPU oracle for the VeLoRA hot path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes loader around ``velora_oracle.cpp`` (plain C++17, double
precision, written from the paper's Sec. 3.1/3.2 definitions and Listing 1).
Only the tests, the smoke check and the benchmark's ``cpu_baseline`` leg may
import this package; the product package never does.

Arrays are numpy: float32 storage is ``np.float32``; bfloat16 storage is
``np.uint16`` bit patterns.  ``M`` is the number of sub-tokens per token and
``d = D // M`` the sub-token size (the paper writes M for the size).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "velora_oracle.cpp")
_LIB = os.path.join(_HERE, "libvelora_oracle.so")

DT_F32 = 0
DT_BF16 = 1
ERR_DEGENERATE = 6


def build(force: bool = False) -> str:
    """Compile the oracle with the host compiler (no GPU code)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-pthread", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    L = ctypes.CDLL(_LIB)
    i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
    L.velora_oracle_round_bf16.argtypes = [ctypes.c_double]
    L.velora_oracle_round_bf16.restype = ctypes.c_uint16
    L.velora_oracle_widen_bf16.argtypes = [ctypes.c_uint16]
    L.velora_oracle_widen_bf16.restype = ctypes.c_double
    L.velora_oracle_store_array.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_void_p]
    L.velora_oracle_store_array.restype = None
    L.velora_oracle_init_v.argtypes = [vp, ci, i64, i64, i64, vp, vp, ci]
    L.velora_oracle_init_v.restype = ci
    L.velora_oracle_update_v.argtypes = [vp, ci, i64, i64, i64, vp, ctypes.c_double, vp, vp, ci]
    L.velora_oracle_update_v.restype = ci
    L.velora_oracle_compress.argtypes = [vp, ci, vp, i64, i64, i64, vp, vp, ci]
    L.velora_oracle_compress.restype = None
    L.velora_oracle_reconstruct.argtypes = [vp, ci, vp, i64, i64, i64, vp, ci]
    L.velora_oracle_reconstruct.restype = None
    L.velora_oracle_weight_grad_bruteforce.argtypes = [vp, vp, vp, i64, i64, i64, i64, ci, vp, ci]
    L.velora_oracle_weight_grad_bruteforce.restype = None
    L.velora_oracle_weight_grad_bruteforce_rows.argtypes = [vp, vp, vp, i64, i64, i64, i64, ci, vp, i64, vp, ci]
    L.velora_oracle_weight_grad_bruteforce_rows.restype = None
    L.velora_oracle_weight_grad_factored.argtypes = [vp, vp, vp, i64, i64, i64, i64, ci, vp, vp, ci]
    L.velora_oracle_weight_grad_factored.restype = None
    L.velora_oracle_linear.argtypes = [vp, vp, ci, i64, i64, i64, vp, ci]
    L.velora_oracle_linear.restype = None
    _lib = L
    return L


def default_threads() -> int:
    """Host threads the oracle uses: the cores this process may run on, capped
    by OMP_NUM_THREADS when that is set (shared boxes export their CPU share
    there) and by 16 otherwise."""
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:  # pragma: no cover
        n = os.cpu_count() or 1
    try:
        cap = int(os.environ.get("OMP_NUM_THREADS", "16"))
    except ValueError:
        cap = 16
    return max(1, min(n, cap))


def _dt(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return DT_F32
    if a.dtype == np.uint16:
        return DT_BF16
    raise TypeError(f"storage array must be float32 or uint16 (bf16 bits), got {a.dtype}")


def _c(a: np.ndarray) -> np.ndarray:
    if not a.flags["C_CONTIGUOUS"]:
        raise ValueError("array must be C-contiguous")
    return a


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _v32(v: np.ndarray, d: int) -> np.ndarray:
    v = np.ascontiguousarray(v, dtype=np.float32)
    if v.shape != (d,):
        raise ValueError(f"v must have shape ({d},), got {v.shape}")
    return v


def round_bf16(x: float) -> int:
    return int(_load().velora_oracle_round_bf16(float(x)))


def widen_bf16(b: int) -> float:
    return float(_load().velora_oracle_widen_bf16(int(b)))


def init_v(X: np.ndarray, M: int, threads: int = 0) -> Tuple[np.ndarray, np.ndarray, int]:
    """-> (v float32[d], un-normalised mean float64[d], status 0 | 6)."""
    X = _c(X)
    N, D = X.shape
    assert D % M == 0
    d = D // M
    mean = np.empty(d, dtype=np.float64)
    v = np.empty(d, dtype=np.float32)
    rc = _load().velora_oracle_init_v(_p(X), _dt(X), N, D, M, _p(mean), _p(v), threads or default_threads())
    return v, mean, int(rc)


def update_v(X: np.ndarray, M: int, state: Optional[np.ndarray] = None, beta: float = 0.0,
             threads: int = 0) -> Tuple[np.ndarray, Optional[np.ndarray], int]:
    """Per-batch vector.  -> (v float32[d], new state float32[d] or None, status 0 | 6)."""
    X = _c(X)
    N, D = X.shape
    assert D % M == 0
    d = D // M
    v = np.empty(d, dtype=np.float32)
    st_in = None if state is None else _v32(state, d)
    st_out = None if state is None else np.empty(d, dtype=np.float32)
    rc = _load().velora_oracle_update_v(_p(X), _dt(X), N, D, M, _p(st_in), float(beta), _p(st_out), _p(v),
                                        threads or default_threads())
    return v, st_out, int(rc)


def compress(X: np.ndarray, v: np.ndarray, M: int, threads: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """-> (S_exact float64[N, M], S_store in X's storage dtype [N, M])."""
    X = _c(X)
    N, D = X.shape
    assert D % M == 0
    v = _v32(v, D // M)
    S_exact = np.empty((N, M), dtype=np.float64)
    S_store = np.empty((N, M), dtype=X.dtype)
    _load().velora_oracle_compress(_p(X), _dt(X), _p(v), N, D, M, _p(S_exact), _p(S_store),
                                   threads or default_threads())
    return S_exact, S_store


def reconstruct(S: np.ndarray, v: np.ndarray, D: int, threads: int = 0) -> np.ndarray:
    """-> Xhat float64[N, D]."""
    S = _c(S)
    N, M = S.shape
    assert D % M == 0
    v = _v32(v, D // M)
    Xhat = np.empty((N, D), dtype=np.float64)
    _load().velora_oracle_reconstruct(_p(S), _dt(S), _p(v), N, D, M, _p(Xhat), threads or default_threads())
    return Xhat


def weight_grad_bruteforce(G: np.ndarray, S: np.ndarray, v: np.ndarray, D: int, threads: int = 0) -> np.ndarray:
    """dW float64[O, D] = G^T @ ungroup(reconstruct(S, v)), Xhat materialised."""
    G, S = _c(G), _c(S)
    N, O = G.shape
    N2, M = S.shape
    assert N == N2 and _dt(G) == _dt(S) and D % M == 0
    v = _v32(v, D // M)
    dW = np.empty((O, D), dtype=np.float64)
    _load().velora_oracle_weight_grad_bruteforce(_p(G), _p(S), _p(v), N, O, D, M, _dt(G), _p(dW),
                                                 threads or default_threads())
    return dW


def weight_grad_bruteforce_rows(G: np.ndarray, S: np.ndarray, v: np.ndarray, D: int,
                                rows: Sequence[int], threads: int = 0) -> np.ndarray:
    """Rows ``rows`` of the brute-force dW, float64[len(rows), D]."""
    G, S = _c(G), _c(S)
    N, O = G.shape
    N2, M = S.shape
    assert N == N2 and _dt(G) == _dt(S) and D % M == 0
    v = _v32(v, D // M)
    r = np.ascontiguousarray(rows, dtype=np.int64)
    assert r.ndim == 1 and (r >= 0).all() and (r < O).all()
    out = np.empty((r.shape[0], D), dtype=np.float64)
    _load().velora_oracle_weight_grad_bruteforce_rows(_p(G), _p(S), _p(v), N, O, D, M, _dt(G), _p(r),
                                                      r.shape[0], _p(out), threads or default_threads())
    return out


def weight_grad_factored(G: np.ndarray, S: np.ndarray, v: np.ndarray, D: int,
                         threads: int = 0, want_dW: bool = True) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    """-> (T float64[O, M], dW float64[O, D] or None)."""
    G, S = _c(G), _c(S)
    N, O = G.shape
    N2, M = S.shape
    assert N == N2 and _dt(G) == _dt(S) and D % M == 0
    v = _v32(v, D // M)
    T = np.empty((O, M), dtype=np.float64)
    dW = np.empty((O, D), dtype=np.float64) if want_dW else None
    _load().velora_oracle_weight_grad_factored(_p(G), _p(S), _p(v), N, O, D, M, _dt(G), _p(T), _p(dW),
                                               threads or default_threads())
    return T, dW


def linear(X: np.ndarray, W: np.ndarray, threads: int = 0) -> np.ndarray:
    """Y float64[N, O] = X @ W^T with W stored [O, D]."""
    X, W = _c(X), _c(W)
    N, D = X.shape
    O, D2 = W.shape
    assert D == D2 and _dt(X) == _dt(W)
    Y = np.empty((N, O), dtype=np.float64)
    _load().velora_oracle_linear(_p(X), _p(W), _dt(X), N, D, O, _p(Y), threads or default_threads())
    return Y


def _store(x: np.ndarray, dt: int) -> np.ndarray:
    """float64 -> storage dtype in ONE rounding to nearest even (float32, or bfloat16 bits by the same
    routine as round_bf16): the stored value of Listing 1's `out` and `grad_input` in the training dtype."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    out = np.empty(x.shape, dtype=np.uint16 if dt == DT_BF16 else np.float32)
    _load().velora_oracle_store_array(_p(x), dt, x.size, _p(out))
    return out


def linear_compress(X: np.ndarray, W: np.ndarray, v: np.ndarray, M: int,
                    threads: int = 0) -> Tuple[np.ndarray, np.ndarray, np.ndarray, np.ndarray]:
    """Listing 1's forward as one call: the dense product Y = X @ W^T (W stored
    [O, D]; the listing leaves the dense product as it is) and, next to it, Sec. 3.1's compress of
    the same X, which is what the layer keeps for backward.  Both from their
    definitions in float64, then stored in the inputs' dtype.
    -> (Y_exact float64[N, O], Y_store storage[N, O], S_exact float64[N, M], S_store storage[N, M])
    """
    Y_exact = linear(X, W, threads=threads)
    S_exact, S_store = compress(X, v, M, threads=threads)
    return Y_exact, _store(Y_exact, _dt(_c(X))), S_exact, S_store


def grad_input(G: np.ndarray, W: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Listing 1, backward: grad_input = grad_output @ weight, dX[n, c] = sum_o G[n, o] * W[o, c]
    with W stored [O, D]; float64 (numpy's matmul on the widened inputs), then stored in the inputs' dtype.
    -> (dX_exact float64[N, D], dX_store storage[N, D])"""
    G, W = _c(G), _c(W)
    assert G.shape[1] == W.shape[0] and _dt(G) == _dt(W)
    if _dt(G) == DT_BF16:
        g = (G.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        w = (W.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    else:
        g, w = G.astype(np.float64), W.astype(np.float64)
    dX = g @ w
    return dX, _store(dX, _dt(G))


def adamw_step_factor(T: np.ndarray, v: np.ndarray, W: np.ndarray, exp_avg: np.ndarray, exp_avg_sq: np.ndarray,
                      lr: float, beta1: float, beta2: float, eps: float, weight_decay: float, step: int,
                      grad_scale: float = 1.0) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """One AdamW step (the optimiser of the paper's training set-ups, Sec. 4.1;
    decoupled weight decay, bias-corrected moments) on a weight whose gradient is
    given in the factored form of Sec. 3.1's reconstruction,
    dW[o, g*d + j] = grad_scale * T[o, g] * v[j].  Everything in float64:

        W   <- W * (1 - lr * weight_decay)
        m   <- beta1 * m + (1 - beta1) * dW
        u   <- beta2 * u + (1 - beta2) * dW^2
        W   <- W - lr / (1 - beta1^step) * m / (sqrt(u) / sqrt(1 - beta2^step) + eps)

    W float64[O, D] (widen bf16 storage before calling), m = exp_avg, u = exp_avg_sq
    float64[O, D], step >= 1.  -> (W_new, m_new, u_new), float64, inputs untouched.
    """
    T = np.asarray(T, dtype=np.float64)
    vv = np.asarray(v, dtype=np.float64).reshape(1, -1)
    W = np.asarray(W, dtype=np.float64)
    m = np.asarray(exp_avg, dtype=np.float64)
    u = np.asarray(exp_avg_sq, dtype=np.float64)
    O, M = T.shape
    d = vv.shape[1]
    assert W.shape == (O, M * d) and m.shape == W.shape and u.shape == W.shape and step >= 1
    dW = float(grad_scale) * np.kron(T, vv)           # [O, M*d], column g*d + j holds T[o, g] * v[j]
    W1 = W * (1.0 - lr * weight_decay)
    m1 = beta1 * m + (1.0 - beta1) * dW
    u1 = beta2 * u + (1.0 - beta2) * dW * dW
    bc1 = 1.0 - beta1 ** step
    bc2 = 1.0 - beta2 ** step
    W2 = W1 - (lr / bc1) * m1 / (np.sqrt(u1) / np.sqrt(bc2) + eps)
    return W2, m1, u1


def swiglu_compress(gate: np.ndarray, up: np.ndarray, v: np.ndarray, M: int,
                    threads: int = 0) -> Tuple[np.ndarray, np.ndarray, np.ndarray, np.ndarray]:
    """The input of an LLaMA-style down projection, produced and compressed in one
    go: X = silu(gate) * up with silu(x) = x / (1 + exp(-x)) (float64), stored in the
    inputs' dtype (one round-to-nearest-even for bfloat16); then Sec. 3.1's
    compress applied to the STORED X, exactly as `compress` would be applied to it
    afterwards.  gate, up: [N, D] storage arrays of one dtype.
    -> (X_exact float64[N, D], X_store storage[N, D], S_exact float64[N, M], S_store storage[N, M])
    """
    gate, up = _c(gate), _c(up)
    assert gate.shape == up.shape and _dt(gate) == _dt(up)
    if _dt(gate) == DT_BF16:
        g = (gate.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        u = (up.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    else:
        g, u = gate.astype(np.float64), up.astype(np.float64)
    X_exact = g / (1.0 + np.exp(-g)) * u
    if _dt(gate) == DT_BF16:
        f = X_exact.astype(np.float32)                      # float64 -> float32 -> bfloat16: the double
        b = f.view(np.uint32)                               # rounding can differ from a single one only in
        lsb = (b >> 16) & 1                                 # ties that float32 cannot represent apart
        X_store = ((b + 0x7FFF + lsb) >> 16).astype(np.uint16)
    else:
        X_store = X_exact.astype(np.float32)
    S_exact, S_store = compress(X_store, v, M, threads=threads)
    return X_exact, X_store, S_exact, S_store


def rmsnorm_compress(H: np.ndarray, gamma: np.ndarray, eps: float, v: np.ndarray, M: int,
                     threads: int = 0) -> Tuple[np.ndarray, np.ndarray, np.ndarray, np.ndarray]:
    """The input of an LLaMA-style attention projection, produced and compressed in
    one go: X[n, :] = H[n, :] / sqrt(mean_j H[n, j]^2 + eps) * gamma (float64),
    stored in H's dtype (one round-to-nearest-even for bfloat16); then Sec. 3.1's
    compress applied to the STORED X.  H: [N, D] storage array; gamma: float32 [D].
    -> (X_exact float64[N, D], X_store storage[N, D], S_exact float64[N, M], S_store storage[N, M])
    """
    H = _c(H)
    if _dt(H) == DT_BF16:
        h = (H.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    else:
        h = H.astype(np.float64)
    g = np.asarray(gamma, dtype=np.float32).astype(np.float64).reshape(1, -1)
    assert g.shape[1] == h.shape[1]
    ms = (h * h).mean(axis=1, keepdims=True)
    X_exact = h / np.sqrt(ms + float(eps)) * g
    if _dt(H) == DT_BF16:
        b = X_exact.astype(np.float32).view(np.uint32)
        X_store = ((b + 0x7FFF + ((b >> 16) & 1)) >> 16).astype(np.uint16)
    else:
        X_store = X_exact.astype(np.float32)
    S_exact, S_store = compress(X_store, v, M, threads=threads)
    return X_exact, X_store, S_exact, S_store
