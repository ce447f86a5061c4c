"""The seeded input generators: determinism, shapes and statistics."""
import numpy as np
import pytest

import workloads as wl


def test_shape_table_matches_configs():
    names = [s.name for s in wl.all_shapes()]
    assert len(names) == len(set(names))
    s = wl.shape_by_name("cfg1_tiny")
    assert (s.N, s.D, s.O, s.d, s.M, s.dtype, s.seed) == (256, 64, 64, 16, 4, wl.F32, 0)
    s = wl.shape_by_name("cfg2_vit_fc1")
    assert (s.N, s.D, s.O, s.d, s.M) == (64 * 197, 768, 3072, 64, 12)
    s = wl.shape_by_name("cfg3_down")
    assert (s.N, s.D, s.O, s.d, s.M) == (65536, 2048, 768, 128, 16)
    s = wl.shape_by_name("cfg4_down")
    assert (s.N, s.D, s.O, s.d, s.M) == (16384, 11008, 4096, 256, 43)
    s = wl.shape_by_name("cfg5_down_d64")
    assert (s.N, s.D, s.O, s.d, s.M) == (16384, 13824, 5120, 64, 216)
    bad = wl.shape_by_name("cfg5_down_d1024")
    assert not bad.divisible and bad not in wl.valid_shapes()
    assert wl.shape_by_name("cfg5_down_d512").M == 27


def test_bf16_conversion_roundtrip_and_rne():
    b = np.arange(0, 1 << 16, dtype=np.uint32).astype(np.uint16)
    f = wl.bf16_bits_to_f32(b)
    ok = ~np.isnan(f)
    assert (wl.f32_to_bf16_bits(f[ok]) == b[ok]).all()
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20], dtype=np.float32)
    assert list(wl.f32_to_bf16_bits(x)) == [0x3F80, 0x3F82, 0x3F81]


@pytest.mark.parametrize("name", ["cfg1_tiny", "cfg2_vit_fc1"])
def test_deterministic(name):
    sh = wl.reduced(wl.shape_by_name(name), 64)
    assert (wl.make_X(sh) == wl.make_X(sh)).all()
    assert (wl.make_G(sh) == wl.make_G(sh)).all()


def test_distributions():
    sh = wl.reduced(wl.shape_by_name("cfg2_vit_fc1"), 4096)
    X = wl.to_f64(wl.make_X(sh), sh.dtype)
    col_std = X.std(axis=0)
    assert 0.45 < col_std.min() and col_std.max() < 2.2 and col_std.max() / col_std.min() > 2.5
    G = wl.to_f64(wl.make_G(sh), sh.dtype)
    assert abs(G.std() - 0.02) < 5e-4

    sh = wl.reduced(wl.shape_by_name("cfg4_attn"), 2048)
    X = wl.to_f64(wl.make_X(sh), sh.dtype)
    assert abs(X.var() - 1.0) < 0.1                      # t_4 / sqrt(2) has unit variance
    kurt = (X ** 4).mean() / X.var() ** 2
    assert kurt > 6.0                                     # far heavier tails than a Gaussian (3)

    sh = wl.reduced(wl.shape_by_name("cfg5_attn_d64"), 2048)
    X = wl.to_f64(wl.make_X(sh), sh.dtype)
    col_std = X.std(axis=0)
    n_out = int((col_std > 10).sum())
    assert n_out == round(0.01 * sh.D) == 51
    assert abs(np.median(col_std) - 1.0) < 0.05


def test_random_unit_v():
    v = wl.random_unit_v(256, 3)
    assert v.dtype == np.float32 and abs(np.linalg.norm(v.astype(np.float64)) - 1) < 1e-6


def test_two_bfloat16_parts_carry_a_float32_to_17_bits():
    """The GEMM that forms S inside its own tiles (velora_linear_compress) feeds v to the matrix
    pipes as hi + lo, two bfloat16 numbers: hi = bf16(v), lo = bf16(v - hi).  The stated bound
    |v - hi - lo| <= 2^-17 |v| is arithmetic, checked here with the generators' own rounding."""
    rng = np.random.default_rng(11)
    v = np.concatenate([rng.standard_normal(20000), rng.standard_normal(2000) * 1e-6,
                        np.array([1.0, -1.0, 0.0, 1.0 + 2.0 ** -8, 3.0 - 2.0 ** -7])]).astype(np.float32)
    hi = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(v))
    lo = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits((v - hi).astype(np.float32)))
    err = np.abs(v.astype(np.float64) - hi.astype(np.float64) - lo.astype(np.float64))
    assert (err <= 2.0 ** -17 * np.abs(v.astype(np.float64))).all()
