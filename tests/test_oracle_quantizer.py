"""Pins for the oracle's quantiser (paper Sec. 3.2.1: asymmetric groupwise
quantisation, G = 32, one (scale, zero-point) pair per group).

Nothing here re-types the oracle's formula: the pins are hand-worked groups
(tests/golden/quant_worked_groups.txt), numpy's own fp16 casts and division
for the stored scale / zero, an exact-arithmetic nearest-code search, and the
scale/2 round-trip bound."""
import os
from fractions import Fraction

import numpy as np
import pytest

from paper_2605_17170_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden", "quant_worked_groups.txt")


def _load_cases():
    cases, cur = [], None
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line.startswith("case "):
            parts = line.split()
            cur = {"name": parts[1]}
            for p in parts[2:]:
                k, v = p.split("=")
                cur[k] = int(v, 16) if k in ("scale", "zero") else int(v)
            cases.append(cur)
        elif line.startswith("x:"):
            cur["x"] = [float(v) for v in line[2:].split()]
        elif line.startswith("c:"):
            cur["c"] = [int(v) for v in line[2:].split()]
    return cases


@pytest.mark.parametrize("case", _load_cases(), ids=lambda c: c["name"])
def test_worked_groups(oracle, case):
    assert len(case["x"]) == 32 and len(case["c"]) == 32
    x = np.float32(case["x"])
    xb = wl.f32_to_bf16_bits(x)
    assert np.array_equal(wl.bf16_bits_to_f32(xb), x), "fixture values must be bf16-exact"
    codes, s, z = oracle.quantize_group(xb, case["bits"])
    assert s == case["scale"] and z == case["zero"]
    assert codes.tolist() == case["c"]


def _random_groups(rng, n, kind):
    x = rng.standard_normal((n, 32)).astype(np.float32)
    if kind == "outlier":
        x[np.arange(n), rng.integers(0, 32, n)] *= 20
    elif kind == "tiny":
        x *= np.float32(2.0) ** rng.integers(-20, -8, (n, 1)).astype(np.float32)
    elif kind == "shifted":
        x = x * np.float32(0.01) + rng.uniform(-50, 50, (n, 1)).astype(np.float32)
    elif kind == "halves":
        x = np.round(x * 4) / 4
    return wl.f32_to_bf16_bits(x)


@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("kind", ["normal", "outlier", "tiny", "shifted", "halves"])
def test_scale_zero_match_numpy_casts(oracle, bits, kind):
    """zero = fp16(min) and scale = fp16((max-min)/L) with the casts and the
    fp32 division done by numpy."""
    rng = np.random.default_rng(100 + bits)
    xb = _random_groups(rng, 2000, kind)
    x = wl.bf16_bits_to_f32(xb)
    L = np.float32(2 ** bits - 1)
    for i in range(xb.shape[0]):
        _, s, z = oracle.quantize_group(xb[i], bits)
        mn, mx = x[i].min(), x[i].max()
        with np.errstate(over="ignore"):
            want_s = np.float16(np.float32(mx - mn) / L).view(np.uint16)
            want_z = np.float16(mn + np.float32(0.0)).view(np.uint16)
        assert s == int(want_s) and z == int(want_z)


def test_negative_zero_minimum_is_stored_as_plus_zero(oracle):
    x = np.float32([-0.0] + [1.0] * 31)
    xb = wl.f32_to_bf16_bits(x)
    assert xb[0] == 0x8000
    _, s, z = oracle.quantize_group(xb, 4)
    assert z == 0x0000


@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("kind", ["normal", "outlier", "shifted", "halves"])
def test_codes_are_nearest_levels(oracle, bits, kind):
    """Exact-arithmetic check: the emitted code is the level z + c*s nearest
    to x (ties to the even code) whenever x is not within 2^-12 of a
    half-way point in units of s (fp32 rounding of the product may move
    such near-ties)."""
    rng = np.random.default_rng(200 + bits)
    xb = _random_groups(rng, 300, kind)
    x = wl.bf16_bits_to_f32(xb)
    L = 2 ** bits - 1
    checked = 0
    for i in range(xb.shape[0]):
        codes, s, z = oracle.quantize_group(xb[i], bits)
        sf = Fraction(float(np.uint16(s).view(np.float16)))
        zf = Fraction(float(np.uint16(z).view(np.float16)))
        if sf == 0:
            assert not codes.any()
            continue
        for j in range(32):
            t = (Fraction(float(x[i, j])) - zf) / sf
            fl = t.numerator // t.denominator
            frac = t - fl
            if abs(frac - Fraction(1, 2)) < Fraction(1, 4096):
                continue
            c = fl + (1 if frac > Fraction(1, 2) else 0)
            c = min(max(c, 0), L)
            assert codes[j] == c
            checked += 1
    assert checked > 2000


@pytest.mark.parametrize("bits", [2, 4])
def test_exact_ties_go_to_even(oracle, bits):
    """Power-of-two scale, zero 0: (x - z)/s is exact, so k + 0.5 must give
    the even neighbour."""
    L = 2 ** bits - 1
    for s in (0.25, 1.0, 4.0):
        xs = [0.0, L * s] + [(k + 0.5) * s for k in range(L)]
        xs = (xs * 32)[:32]
        xb = wl.f32_to_bf16_bits(np.float32(xs))
        codes, sh, zh = oracle.quantize_group(xb, bits)
        assert np.uint16(sh).view(np.float16) == s and zh == 0
        for v, c in zip(xs, codes):
            k = v / s
            want = int(k) if k == int(k) else (int(k) if int(k) % 2 == 0 else int(k) + 1)
            assert c == want


@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("kind", ["normal", "outlier", "shifted"])
def test_round_trip_error_at_most_half_a_step(oracle, bits, kind):
    """|x - (z + c*s)| <= s/2 (1 + 2^-10) for every element, plus, for the
    top of the range only, the shortfall L*s < max - z caused by rounding the
    scale down to fp16 (at most L * 2^-11 * s).  Holds when (max-min)/L is in
    fp16's normal range and min is fp16-exact, true for all of these inputs
    except `shifted`, whose minimum is rounded: there the bound gains
    |min - fp16(min)|."""
    rng = np.random.default_rng(300 + bits)
    T = 500
    xb = _random_groups(rng, T, kind).reshape(T, 1, 32)
    codes, scale, zero = oracle.quantize(xb, np.full(T, bits, np.uint8), G=32)
    xh = oracle.dequantize(codes, scale, zero, G=32)
    x = wl.bf16_bits_to_f32(xb).astype(np.float64)
    s = scale.view(np.float16).astype(np.float64)[..., 0][..., None]
    z = zero.view(np.float16).astype(np.float64)[..., 0][..., None]
    L = 2 ** bits - 1
    zerr = np.abs(x.min(axis=-1, keepdims=True) - z)
    bound = s / 2 * (1 + 2.0 ** -10) + L * 2.0 ** -11 * s + zerr
    ok = np.broadcast_to(s >= 2.0 ** -14, x.shape)  # the bound is claimed in fp16's normal range only
    assert ok[..., 0].mean() > 0.3
    assert np.all((np.abs(x - xh) <= bound) | ~ok)
    # and the plain scale/2 bound for everything that is not clamped at the top code
    inner = (codes < L) & ok
    assert np.all(np.abs(x - xh)[inner] <= (s / 2 * (1 + 2.0 ** -10) + zerr + 0 * x)[inner])


def test_dequantize_matches_numpy(oracle):
    rng = np.random.default_rng(5)
    T, H, D = 37, 3, 128
    x = wl.normal_bf16(rng, (T, H, D))
    bits = rng.choice([2, 4], T).astype(np.uint8)
    codes, scale, zero = oracle.quantize(x, bits)
    assert codes[bits == 2].max() <= 3 and codes.max() <= 15
    xh = oracle.dequantize(codes, scale, zero)
    s = np.repeat(scale.view(np.float16).astype(np.float64), 32, axis=-1)
    z = np.repeat(zero.view(np.float16).astype(np.float64), 32, axis=-1)
    assert np.array_equal(xh, codes * s + z)


def test_groups_are_independent_and_per_token(oracle):
    """Changing one channel changes codes/scale/zero of its own group only."""
    rng = np.random.default_rng(6)
    x = wl.normal_bf16(rng, (4, 2, 128))
    bits = np.uint8([2, 4, 2, 4])
    a = oracle.quantize(x, bits)
    y = x.copy()
    y[2, 1, 70] = wl.f32_to_bf16_bits(np.float32([123.0]))[0]
    b = oracle.quantize(y, bits)
    diff = np.zeros((4, 2, 4), bool)
    diff[2, 1, 70 // 32] = True
    for u, v in zip(a[1:], b[1:]):
        assert np.array_equal(u != v, diff & (u != v))
    changed = (a[0] != b[0]).reshape(4, 2, 4, 32).any(-1)
    assert changed[2, 1, 2] and changed.sum() == 1


def test_bad_bitwidth_is_rejected(oracle):
    x = np.zeros((2, 1, 128), np.uint16)
    with pytest.raises(ValueError):
        oracle.quantize(x, np.uint8([2, 3]))
