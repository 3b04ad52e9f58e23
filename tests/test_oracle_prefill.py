"""Pins of the oracle's FP16 dequantisation (prefill gather, Sec. 3.2.3 "Prefill").

The conversion is pinned against numpy's float64 -> float16 cast (an independent library routine) and
the dequantised values against exact rational arithmetic with a rounding routine written here for the
test; a detour through binary32 (two roundings) is shown to be a different function, so a mistake of that
kind in the oracle would fail.
"""
import warnings
from fractions import Fraction

import numpy as np
import pytest

from paper_2605_17170_amd import workloads as wl


def _f16_values():
    """Every finite binary16 value as a Fraction, ascending, with its bit pattern."""
    bits = np.arange(0, 0x7c00, dtype=np.uint16)
    vals = [Fraction(float(v)) for v in bits.view(np.float16)]
    return bits, vals


def _round_fraction_to_f16(x: Fraction, bits, vals) -> int:
    """Nearest-even binary16 bit pattern of an exact rational (brute force over the value table)."""
    sign = 0x8000 if x < 0 else 0
    a = abs(x)
    if a >= Fraction(65520):
        return sign | 0x7c00
    lo, hi = 0, len(vals) - 1
    while lo < hi:                      # largest value <= a
        mid = (lo + hi + 1) // 2
        if vals[mid] <= a:
            lo = mid
        else:
            hi = mid - 1
    if lo == len(vals) - 1:
        up_val = Fraction(65536)        # the value binary16 would have with one more exponent
        down, up = vals[lo], up_val
        choose_up = (a - down > up - a) or (a - down == up - a and (int(bits[lo]) & 1))
        return sign | (0x7c00 if choose_up else int(bits[lo]))
    down, up = vals[lo], vals[lo + 1]
    if a - down < up - a:
        return sign | int(bits[lo])
    if a - down > up - a:
        return sign | int(bits[lo + 1])
    return sign | int(bits[lo] if (int(bits[lo]) & 1) == 0 else bits[lo + 1])


def test_f64_to_f16_matches_numpy_cast(oracle):
    rng = np.random.default_rng(5)
    parts = [
        rng.standard_normal(200000) * 10.0 ** rng.integers(-9, 6, 200000),
        np.array([0.0, -0.0, 65504.0, 65519.999, 65520.0, 1e9, -1e9, np.inf, -np.inf, 2.0 ** -24, 2.0 ** -25,
                  2.0 ** -25 * (1 + 2.0 ** -40), 2.0 ** -26, 6.1e-5, 6.097555160522461e-05]),
    ]
    # exact ties and their neighbours: odd multiples of half an ulp, +- one binary64 ulp
    h = np.arange(1, 0x7bff, 7, dtype=np.uint16).view(np.float16).astype(np.float64)
    nxt = np.arange(2, 0x7c00, 7, dtype=np.uint16).view(np.float16).astype(np.float64)
    mid = (h + nxt) / 2
    parts += [mid, np.nextafter(mid, np.inf), np.nextafter(mid, -np.inf), -mid]
    x = np.concatenate(parts)
    with warnings.catch_warnings():
        warnings.simplefilter("ignore")
        want = x.astype(np.float16).view(np.uint16)
    assert np.array_equal(oracle.f64_to_f16(x), want)
    nan = oracle.f64_to_f16(np.array([np.nan]))
    assert (nan[0] & 0x7c00) == 0x7c00 and (nan[0] & 0x3ff) != 0


def test_one_rounding_differs_from_two(oracle):
    """1 + 2^-11 + 2^-30 rounds up in one step but to even (down) after a binary32 detour."""
    x = np.array([1 + 2.0 ** -11 + 2.0 ** -30])
    assert oracle.f64_to_f16(x)[0] == 0x3c01
    assert oracle.f32_to_f16(x.astype(np.float32))[0] == 0x3c00


@pytest.mark.parametrize("bits", [2, 4])
def test_dequantize_f16_is_the_exact_value_rounded_once(oracle, bits):
    rng = np.random.default_rng(30 + bits)
    tb, tv = _f16_values()
    T, H, D = 6, 2, 128
    codes = rng.integers(0, 2 ** bits, (T, H, D)).astype(np.uint8)
    # scales and zeros over the whole binary16 range, including subnormal scales and negative zeros
    scale = rng.integers(0, 0x7000, (T, H, 4)).astype(np.uint16)
    zero = (rng.integers(0, 0x7000, (T, H, 4)) | (rng.integers(0, 2, (T, H, 4)) << 15)).astype(np.uint16)
    got = oracle.dequantize_f16(codes, scale, zero)
    sf = scale.view(np.float16).astype(np.float64)
    zf = zero.view(np.float16).astype(np.float64)
    for t in range(T):
        for h in range(H):
            for c in range(0, D, 3):
                exact = Fraction(int(codes[t, h, c])) * Fraction(float(sf[t, h, c // 32])) + Fraction(float(zf[t, h, c // 32]))
                want = _round_fraction_to_f16(exact, tb, tv)
                if exact == 0:
                    want &= 0x7fff      # the sign of an exact zero is not pinned here
                    assert (int(got[t, h, c]) & 0x7fff) == want
                else:
                    assert int(got[t, h, c]) == want, (t, h, c)


def test_exactly_representable_cache_dequantises_to_its_source(oracle):
    """Values on a power-of-two grid that the quantiser reproduces: FP16 rows equal the bf16 inputs."""
    rng = np.random.default_rng(33)
    T, H = 40, 2
    bits = rng.choice([2, 4], T).astype(np.uint8)
    vals = np.empty((T, H, 128))
    for b, (z, s) in ((2, (-1.0, 0.5)), (4, (-2.0, 0.25))):
        n = int((bits == b).sum())
        c = rng.integers(0, 2 ** b, (n, H, 4, 32))
        c[..., 0] = 0
        c[..., 1] = 2 ** b - 1
        vals[bits == b] = (z + s * rng.permuted(c, axis=-1)).reshape(n, H, 128)
    x = wl.f32_to_bf16_bits(vals.astype(np.float32))
    q = oracle.quantize(x, bits)
    got = oracle.dequantize_f16(*q).view(np.float16).astype(np.float64)
    assert np.array_equal(got, vals)


def test_dequantize_f16_agrees_with_fp64_dequantisation_to_half_an_ulp(oracle):
    rng = np.random.default_rng(34)
    K, _, _ = wl.make_kv(np.random.SeedSequence(35), 300, 2)
    bits = rng.choice([2, 4], 300).astype(np.uint8)
    q = oracle.quantize(K, bits)
    exact = oracle.dequantize(*q)
    h = oracle.dequantize_f16(*q).view(np.float16).astype(np.float64)
    ulp = np.maximum(2.0 ** (np.floor(np.log2(np.maximum(np.abs(exact), 2.0 ** -14))) - 10), 2.0 ** -24)
    assert np.all(np.abs(h - exact) <= ulp / 2)
    # and monotone in the code within a group: a larger code never gives a smaller FP16 value
    codes, scale, zero = q
    order = np.argsort(codes[5, 1, :32], kind="stable")
    assert np.all(np.diff(h[5, 1, :32][order]) >= 0)
