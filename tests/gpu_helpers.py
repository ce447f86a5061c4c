"""Shared plumbing for the GPU parity tests: host<->device conversion and the
error measures the tolerances are stated in."""
from __future__ import annotations

import numpy as np

import workloads as wl

# Tolerances (the benchmark spec): float32 path 1e-5 relative (Frobenius, and max error
# against the largest magnitude); bf16 inputs with float32 accumulation 2e-2
# relative Frobenius.  The secondary bounds below are what the arithmetic should
# really achieve (one rounding to bf16 on store; exact bf16 products accumulated
# in float32 over N terms, error about sqrt(N) * 2^-24) and are asserted as well.
TOL_F32 = 1e-5
TOL_BF16 = 2e-2
TOL_BF16_STORE = 4e-3        # one RNE rounding to bf16: rms relative error 2^-9/sqrt(3) ~ 1.1e-3
TOL_F32_FROM_BF16 = 2e-5     # float32 results computed from bf16 inputs (exact products, f32 accumulate)


def to_dev(a: np.ndarray, dtype: str):
    import torch
    t = torch.from_numpy(a)
    if dtype == wl.BF16:
        t = t.view(torch.bfloat16)
    return t.cuda()


def to_host_bits(t) -> np.ndarray:
    """GPU tensor -> numpy storage array (float32, or uint16 bf16 bits)."""
    import torch
    if t.dtype == torch.bfloat16:
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return t.contiguous().cpu().numpy()


def to_host_f64(t) -> np.ndarray:
    import torch
    if t.dtype == torch.bfloat16:
        return wl.to_f64(to_host_bits(t), wl.BF16)
    return t.contiguous().cpu().numpy().astype(np.float64)


def rel_fro(a: np.ndarray, b: np.ndarray) -> float:
    nb = float(np.linalg.norm(b))
    return float(np.linalg.norm(a - b)) / (nb if nb > 0 else 1.0)


def rel_max(a: np.ndarray, b: np.ndarray) -> float:
    mb = float(np.abs(b).max())
    return float(np.abs(a - b).max()) / (mb if mb > 0 else 1.0)


def bf16_ordered(bits: np.ndarray) -> np.ndarray:
    """Map bf16 bit patterns to integers that are monotonic in the value."""
    b = bits.astype(np.int32)
    return np.where(b & 0x8000, -(b & 0x7FFF), b)


def assert_bf16_store_matches(gpu_bits: np.ndarray, exact: np.ndarray, ref_bits: np.ndarray, what: str):
    """A value accumulated in float32 and rounded once to bf16 against the
    oracle's double-precision value rounded once to bf16: identical except
    where the exact value sits within float32 accumulation error of a rounding
    boundary (then one bf16 ulp apart), or is so close to zero that its bf16
    ulp is below that error (then a small absolute error)."""
    rms = float(np.sqrt(np.mean(exact * exact))) or 1.0
    big = np.abs(exact) >= 1e-3 * rms
    dist = np.abs(bf16_ordered(gpu_bits) - bf16_ordered(ref_bits))
    assert dist[big].max(initial=0) <= 1, f"{what}: more than one bf16 ulp from the oracle"
    frac = float((dist[big] != 0).mean()) if big.any() else 0.0
    assert frac <= 2e-2, f"{what}: {frac:.2e} of the values differ from the oracle's rounding"
    small_err = np.abs(wl.bf16_bits_to_f32(gpu_bits).astype(np.float64) - exact)[~big]
    assert small_err.max(initial=0.0) <= 5e-5 * rms, f"{what}: error near zero"
