"""Pins of the oracle's E4M3 codec (the 8-bit storage of the compressed cache, an extension of the
decode step of Sec. 4.3) to things other than itself: the values the OCP 8-bit floating point
specification fixes, PyTorch's own float8_e4m3fn cast, exact rational arithmetic for the ties."""
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle

ALL = np.arange(256, dtype=np.uint8)


def test_values_the_format_fixes():
    # sign . exponent(4, bias 7) . mantissa(3); no infinities, S.1111.111 is NaN
    fixed = {0x00: 0.0, 0x38: 1.0, 0x3C: 1.5, 0x40: 2.0, 0x01: 2.0 ** -9, 0x07: 7 * 2.0 ** -9, 0x08: 2.0 ** -6,
             0x7E: 448.0, 0x77: 1.875 * 2 ** 7, 0xB8: -1.0, 0xFE: -448.0, 0x81: -(2.0 ** -9)}
    for code, val in fixed.items():
        assert oracle.e4m3_decode(np.uint8(code)) == val, hex(code)
    assert np.isnan(oracle.e4m3_decode(np.uint8(0x7F))) and np.isnan(oracle.e4m3_decode(np.uint8(0xFF)))
    z = oracle.e4m3_decode(np.uint8(0x80))
    assert z == 0.0 and np.signbit(z)
    assert oracle.E4M3_MAX == 448.0


def test_decode_of_every_code_equals_the_library_cast():
    mine = oracle.e4m3_decode(ALL)
    lib = torch.from_numpy(ALL.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(np.isnan(mine), np.isnan(lib))
    ok = ~np.isnan(mine)
    assert np.array_equal(mine[ok], lib[ok]) and np.array_equal(np.signbit(mine[ok]), np.signbit(lib[ok]))


def test_every_code_survives_a_round_trip_and_the_order_is_monotone():
    ok = (ALL & 0x7F) != 0x7F
    vals = oracle.e4m3_decode(ALL[ok])
    assert np.array_equal(oracle.e4m3_encode(vals.astype(np.float32)), ALL[ok])
    pos = oracle.e4m3_decode(np.arange(0x00, 0x7F, dtype=np.uint8))
    assert (np.diff(pos) > 0).all()
    x = np.sort(np.random.default_rng(0).uniform(-500, 500, 20000).astype(np.float32))
    v = oracle.e4m3_decode(oracle.e4m3_encode(x))
    assert (np.diff(v) >= 0).all()


def test_rounding_is_to_nearest_with_ties_to_even_by_exact_arithmetic():
    # for every pair of neighbouring magnitudes: the midpoint goes to the even code, anything strictly inside a half goes
    # to that half's end.  Everything here is exact (dyadic rationals that binary32 holds).
    for code in range(0x00, 0x7E):
        lo, hi = Fraction(float(oracle.e4m3_decode(np.uint8(code)))), Fraction(float(oracle.e4m3_decode(np.uint8(code + 1))))
        mid = (lo + hi) / 2
        even = code if code % 2 == 0 else code + 1
        assert oracle.e4m3_encode(np.float32(float(mid))) == even, hex(code)
        eps = (hi - lo) / 64
        assert oracle.e4m3_encode(np.float32(float(mid - eps))) == code
        assert oracle.e4m3_encode(np.float32(float(mid + eps))) == code + 1
        assert oracle.e4m3_encode(np.float32(-float(mid))) == (even | 0x80)


def test_nearest_value_by_brute_force():
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.standard_normal(4000) * s for s in (1e-3, 1e-2, 1, 30, 300)]).astype(np.float32)
    x = np.clip(x, -448, 448)
    grid = oracle.e4m3_decode(np.arange(0x00, 0x7F, dtype=np.uint8))          # non-negative finite values, ascending
    d = np.abs(np.abs(x.astype(np.float64))[:, None] - grid[None, :])
    got = oracle.e4m3_decode(oracle.e4m3_encode(x))
    assert np.array_equal(np.abs(np.abs(got) - np.abs(x.astype(np.float64))), d.min(axis=1))
    assert np.array_equal(np.signbit(got), np.signbit(x))


def test_encode_equals_the_library_cast_inside_the_range():
    rng = np.random.default_rng(2)
    x = np.concatenate([rng.standard_normal(50000) * s for s in (2e-3, 0.05, 1, 20, 200)] + [
        np.array([0.0, -0.0, 448.0, -448.0, 447.9, 2.0 ** -10, 2.0 ** -10 * 1.0001, 2.0 ** -9, 1.0625, 1.1875])])
    x = np.clip(x.astype(np.float32), -448, 448)
    lib = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(oracle.e4m3_encode(x), lib)


def test_out_of_range_values_saturate():
    x = np.array([449.0, 464.0, 480.0, 1e6, 3.4e38, np.inf, -449.0, -1e6, -np.inf], dtype=np.float32)
    want = np.array([0x7E] * 6 + [0xFE] * 3, dtype=np.uint8)
    assert np.array_equal(oracle.e4m3_encode(x), want)
    assert oracle.e4m3_encode(np.float32(np.nan)) & 0x7F == 0x7F


def test_quantisation_divides_in_binary32():
    # x = fl32(T * c) with T a tie point (1.0625, halfway between 1.0 and 1.125): the exact quotient x / c misses T by
    # less than half a binary32 ulp, so the binary32 quotient IS T and rounds to the even neighbour 1.0 (code 0x38),
    # whichever side of T the exact quotient lies on.  A division carried out in higher precision would send the
    # cases above T to 1.125 (0x39).
    T = np.float32(1.0625)
    above = 0
    for c in np.float32([1.1, 0.3, 2.7, 0.013, 37.7, 5.3, 0.77]):
        x = np.float32(T * c)
        exact = Fraction(float(x)) / Fraction(float(c))
        assert np.float32(x / c) == T
        above += exact > Fraction(float(T))
        assert oracle.quantize_e4m3(np.full((1, 1, 1), x), [c])[0, 0, 0] == 0x38
    assert above >= 1      # the series does contain cases that tell the two precisions apart


def test_quantise_then_dequantise_per_head_scales():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((2, 3, 5, 8)).astype(np.float32)
    scale = np.float32([0.01, 0.5, 2.0])
    codes = oracle.quantize_e4m3(x, scale)
    back = oracle.dequantize_e4m3(codes, scale)
    for h in range(3):
        y = x[:, h] / scale[h]
        lib = torch.from_numpy(np.clip(y, -448, 448)).to(torch.float8_e4m3fn)
        assert np.array_equal(codes[:, h], lib.view(torch.uint8).numpy())
        assert np.array_equal(back[:, h], lib.to(torch.float64).numpy() * float(scale[h]))
    # relative error of a value well inside the range: at most half a mantissa step, 2^-4
    big = np.abs(x / scale[:, None, None]) >= 2.0 ** -6
    assert (np.abs(back - x)[big] <= np.abs(x)[big] * 2.0 ** -4 * (1 + 1e-6)).all()


def test_decode_on_codes_is_decode_on_the_dequantised_cache():
    rng = np.random.default_rng(4)
    B, Hq, Hkv, Lk, D = 2, 4, 2, 37, 16
    q = rng.standard_normal((B, Hq, D))
    k = rng.standard_normal((B, Hkv, Lk, D)).astype(np.float32)
    v = rng.standard_normal((B, Hkv, Lk, D)).astype(np.float32)
    ks, vs = np.float32([0.02, 0.03]), np.float32([0.015, 0.04])
    kc, vc = oracle.quantize_e4m3(k, ks), oracle.quantize_e4m3(v, vs)
    out, lse = oracle.decode_e4m3(q, kc, vc, ks, vs, seqlens=[37, 20])
    # written out for one (b, h): softmax over the dequantised keys of its sequence
    b, h, n = 1, 3, 20
    kd = oracle.e4m3_decode(kc[b, 1, :n]) * float(ks[1])
    vd = oracle.e4m3_decode(vc[b, 1, :n]) * float(vs[1])
    s = kd @ q[b, h] / np.sqrt(D)
    p = np.exp(s - s.max())
    assert np.allclose(out[b, h], (p / p.sum()) @ vd, rtol=1e-12, atol=1e-14)
    assert np.isclose(lse[b, h], s.max() + np.log(p.sum()), rtol=1e-12)
    # quantisation error of the result is small at these scales
    o0, _ = oracle.decode(q, k.astype(np.float64), v.astype(np.float64), [37, 20])
    assert np.abs(out - o0).max() < 0.1
