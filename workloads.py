"""Seeded synthetic inputs shaped like the paper's ViT and LLaMA linear layers.

This module serves both the CPU oracle and the HIP path and therefore holds
none of the method's arithmetic: it only draws random tensors, rounds them to
the storage dtype and names the layer shapes.  The shapes stand in for the
layers the paper trains (ViT-B/16 on VTAB-1k, LLaMA-130M on C4, LLaMA-7B/13B
on Alpaca; paper Sec. 4 and appendix "Implementation Details"); no dataset
item is used or needed, only the layer geometry and plausible statistics.

Notation (the paper calls the sub-token *size* M; here, as in the library):
    N tokens, D input features, O output features,
    d sub-token size, M = D/d sub-tokens per token.

Every tensor is produced on the host from numpy's counter-based Philox
generator, so the bits are a pure function of (seed, shape, distribution).
bf16 tensors are returned as uint16 bit patterns (numpy has no bf16).
"""
from __future__ import annotations

import concurrent.futures
import os
from dataclasses import dataclass
from typing import List, Optional

import numpy as np

F32 = "f32"
BF16 = "bf16"


# --------------------------------------------------------------------------
# dtype plumbing (format conversion only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even), return uint16 bits."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32)
    rnd = ((bits >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((bits + rnd) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) exactly to float32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(a32: np.ndarray, dtype: str) -> np.ndarray:
    """float32 array -> storage array (float32, or uint16 holding bf16 bits)."""
    if dtype == F32:
        return np.ascontiguousarray(a32, dtype=np.float32)
    if dtype == BF16:
        return f32_to_bf16_bits(a32)
    raise ValueError(f"unknown dtype {dtype!r}")


def to_f64(a: np.ndarray, dtype: str) -> np.ndarray:
    """Storage array -> float64 with exactly the stored values."""
    if dtype == F32:
        return a.astype(np.float64)
    return bf16_bits_to_f32(a).astype(np.float64)


# --------------------------------------------------------------------------
# layer shapes
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Shape:
    """One linear layer's worth of hot-path input."""
    name: str          # unique id, e.g. "cfg4_down_d256"
    cfg: int           # 1..5, index into the benchmark's configs (1-based)
    dtype: str         # storage dtype of X, G and S
    N: int             # tokens (batch x sequence, flattened)
    D: int             # input features
    O: int             # output features
    d: int             # sub-token size
    x_dist: str        # "normal" | "chan_scale" | "student_t4" | "outlier_chan"
    g_sigma: float     # std of the output gradient G ~ N(0, g_sigma)
    seed: int

    @property
    def M(self) -> int:
        return self.D // self.d

    @property
    def divisible(self) -> bool:
        return self.D % self.d == 0

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == F32 else 2

    # algorithmic bytes / flops of the two kernels (dW written as fp32 unless
    # stated otherwise); see the design document for the derivation.
    def compress_bytes(self) -> int:
        b = self.elem_bytes
        return self.N * self.D * b + self.N * self.M * b + 4 * self.d

    def wgrad_bytes(self, dw_bytes: int = 4) -> int:
        b = self.elem_bytes
        return self.N * self.O * b + self.N * self.M * b + self.O * self.D * dw_bytes + 4 * self.d

    def wgrad_flops_factored(self) -> int:
        return 2 * self.N * self.O * self.M + self.O * self.D

    def wgrad_flops_dense(self) -> int:
        return 2 * self.N * self.O * self.D


def _mk(name, cfg, dtype, N, D, O, d, x_dist, g_sigma, tid):
    seed = 0 if cfg == 1 else 1000 * cfg + tid
    return Shape(name, cfg, dtype, N, D, O, d, x_dist, g_sigma, seed)


def all_shapes() -> List[Shape]:
    """Every layer shape of the five configurations (including the one cell
    of configuration 5 whose sub-token size does not divide D), plus three
    layers at the paper's own LLaMA-7B sub-token count (cfg = 6)."""
    s: List[Shape] = []
    s.append(_mk("cfg1_tiny", 1, F32, 256, 64, 64, 16, "normal", 0.02, 0))
    s.append(_mk("cfg2_vit_fc1", 2, BF16, 64 * 197, 768, 3072, 64, "chan_scale", 0.02, 0))
    n3 = 256 * 256
    s.append(_mk("cfg3_qkvo", 3, BF16, n3, 768, 768, 128, "normal", 0.01, 0))
    s.append(_mk("cfg3_up", 3, BF16, n3, 768, 2048, 128, "normal", 0.01, 1))
    s.append(_mk("cfg3_down", 3, BF16, n3, 2048, 768, 128, "normal", 0.01, 2))
    n4 = 8 * 2048
    s.append(_mk("cfg4_attn", 4, BF16, n4, 4096, 4096, 256, "student_t4", 0.005, 0))
    s.append(_mk("cfg4_up", 4, BF16, n4, 4096, 11008, 256, "student_t4", 0.005, 1))
    s.append(_mk("cfg4_down", 4, BF16, n4, 11008, 4096, 256, "student_t4", 0.005, 2))
    n5 = 4 * 4096
    tid = 0
    for d in (64, 256, 1024):
        s.append(_mk(f"cfg5_attn_d{d}", 5, BF16, n5, 5120, 5120, d, "outlier_chan", 0.005, tid)); tid += 1
        s.append(_mk(f"cfg5_up_d{d}", 5, BF16, n5, 5120, 13824, d, "outlier_chan", 0.005, tid)); tid += 1
        s.append(_mk(f"cfg5_down_d{d}", 5, BF16, n5, 13824, 5120, d, "outlier_chan", 0.005, tid)); tid += 1
    # 1024 does not divide 13824; d = 512 keeps the large-d end of the sweep
    # exercised on the down projection.
    s.append(_mk("cfg5_down_d512", 5, BF16, n5, 13824, 5120, 512, "outlier_chan", 0.005, tid))
    # Beyond the five configurations: the paper's own setting for LLaMA-7B, 32 sub-tokens
    # per token ("M = D/32", Sec. 5.2 "Sub-token size", Table 5b), on configuration 4's layers.
    s.append(_mk("paper7b_attn_m32", 6, BF16, n4, 4096, 4096, 128, "student_t4", 0.005, 0))
    s.append(_mk("paper7b_up_m32", 6, BF16, n4, 4096, 11008, 128, "student_t4", 0.005, 1))
    s.append(_mk("paper7b_down_m32", 6, BF16, n4, 11008, 4096, 344, "student_t4", 0.005, 2))
    # the other sub-token counts of the paper's ablation (8, 16, 64 per token) on the same 11008-wide input
    s.append(_mk("paper7b_down_m8", 6, BF16, n4, 11008, 4096, 1376, "student_t4", 0.005, 3))
    s.append(_mk("paper7b_down_m16", 6, BF16, n4, 11008, 4096, 688, "student_t4", 0.005, 4))
    s.append(_mk("paper7b_down_m64", 6, BF16, n4, 11008, 4096, 172, "student_t4", 0.005, 5))
    return s


def valid_shapes() -> List[Shape]:
    return [s for s in all_shapes() if s.divisible]


def shape_by_name(name: str) -> Shape:
    for s in all_shapes():
        if s.name == name:
            return s
    raise KeyError(name)


def reduced(shape: Shape, N: int) -> Shape:
    """Same layer, fewer tokens (for cases the oracle must finish quickly)."""
    return Shape(shape.name + f"_n{N}", shape.cfg, shape.dtype, N, shape.D, shape.O,
                 shape.d, shape.x_dist, shape.g_sigma, shape.seed)


# --------------------------------------------------------------------------
# generators
# --------------------------------------------------------------------------
def _rng(seed: int, stream: int, block: int = 0) -> np.random.Generator:
    """Counter-based generator keyed by (seed, stream) with the row-block index
    in the counter's top word, so every block of rows is an independent,
    reproducible stream whatever the number of worker threads."""
    return np.random.Generator(np.random.Philox(key=[np.uint64(seed), np.uint64(stream)],
                                                counter=[0, 0, 0, np.uint64(block)]))


_ROWS_PER_BLOCK = 256


def _workers() -> int:
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:  # pragma: no cover
        n = os.cpu_count() or 1
    return max(1, min(n, 16))


def _fill_rows(out: np.ndarray, fn) -> None:
    """out[r0:r1] = fn(block_index, n_rows) for consecutive blocks of rows."""
    N = out.shape[0]
    blocks = [(b, r0, min(N, r0 + _ROWS_PER_BLOCK)) for b, r0 in enumerate(range(0, N, _ROWS_PER_BLOCK))]

    def run(item):
        b, r0, r1 = item
        out[r0:r1] = fn(b, r1 - r0)

    if len(blocks) == 1:
        run(blocks[0])
        return
    with concurrent.futures.ThreadPoolExecutor(max_workers=_workers()) as ex:
        list(ex.map(run, blocks))


def make_X(shape: Shape) -> np.ndarray:
    """Activations X[N, D] in storage dtype.

    normal        iid N(0,1)
    chan_scale    N(0,1) times a per-channel scale drawn once from U(0.5, 2)
    student_t4    Student-t with 4 degrees of freedom, divided by sqrt(2) so the
                  variance is 1 (heavy tails)
    outlier_chan  N(0,1) with round(0.01*D) fixed channels multiplied by 20
    """
    N, D = shape.N, shape.D
    aux = _rng(shape.seed, 2)
    scale: Optional[np.ndarray] = None
    if shape.x_dist == "chan_scale":
        scale = aux.uniform(0.5, 2.0, size=D).astype(np.float32)
    elif shape.x_dist == "outlier_chan":
        k = int(round(0.01 * D))
        idx = aux.choice(D, size=k, replace=False)
        scale = np.ones(D, dtype=np.float32)
        scale[idx] = 20.0

    def block(b: int, rows: int) -> np.ndarray:
        rng = _rng(shape.seed, 1, b)
        blk = rng.standard_normal((rows, D), dtype=np.float32)
        if shape.x_dist == "student_t4":
            # t_4 = Z / sqrt(chi2_4 / 4); chi2_4 = 2 * Gamma(shape=2)
            chi = rng.standard_gamma(2.0, size=(rows, D), dtype=np.float32) * np.float32(2.0)
            blk = blk / np.sqrt(chi / np.float32(4.0)) / np.float32(np.sqrt(2.0))
        if scale is not None:
            blk = blk * scale[None, :]
        return to_storage(blk, shape.dtype)

    out = np.empty((N, D), dtype=np.float32 if shape.dtype == F32 else np.uint16)
    _fill_rows(out, block)
    return out


def make_G(shape: Shape) -> np.ndarray:
    """Output gradient G[N, O] ~ N(0, g_sigma) in storage dtype."""
    N, O = shape.N, shape.O

    def block(b: int, rows: int) -> np.ndarray:
        rng = _rng(shape.seed, 3, b)
        blk = rng.standard_normal((rows, O), dtype=np.float32) * np.float32(shape.g_sigma)
        return to_storage(blk, shape.dtype)

    out = np.empty((N, O), dtype=np.float32 if shape.dtype == F32 else np.uint16)
    _fill_rows(out, block)
    return out


def make_W(shape: Shape) -> np.ndarray:
    """Layer weight W[O, D] ~ N(0, 1/sqrt(D)) in storage dtype (for the
    forward linear of the fused linear+compress entry point)."""
    rng = _rng(shape.seed, 4)
    w = rng.standard_normal((shape.O, shape.D), dtype=np.float32) / np.float32(np.sqrt(shape.D))
    return to_storage(w, shape.dtype)


def random_unit_v(d: int, seed: int) -> np.ndarray:
    """A seeded unit vector in float32 (an *input* for tests that do not want
    to depend on init_v)."""
    rng = _rng(seed, 5)
    v = rng.standard_normal(d).astype(np.float64)
    v /= np.sqrt((v * v).sum())
    return v.astype(np.float32)


def random_tensor(rows: int, cols: int, dtype: str, seed: int, stream: int = 6,
                  sigma: float = 1.0) -> np.ndarray:
    """Generic seeded N(0, sigma) matrix in storage dtype (property tests)."""
    rng = _rng(seed, stream)
    a = rng.standard_normal((rows, cols), dtype=np.float32) * np.float32(sigma)
    return to_storage(a, dtype)
