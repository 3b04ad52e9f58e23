"""Pins for the oracle's hand-written number-format code: every conversion is
compared with an independent library cast (numpy float16, torch bfloat16)."""
import numpy as np
import torch


def test_f16_to_f32_exhaustive(oracle):
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.f16_to_f32(bits)
    want = bits.view(np.float16).astype(np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


def test_bf16_to_f32_exhaustive(oracle):
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.bf16_to_f32(bits)
    want = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).to(torch.float32).numpy()
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


def _check_f32_to_f16(oracle, x):
    x = np.ascontiguousarray(x, np.float32)
    x = x[np.isfinite(x)]
    got = oracle.f32_to_f16(x)
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    bad = np.nonzero(got != want)[0]
    assert bad.size == 0, (x[bad[:5]], got[bad[:5]], want[bad[:5]])


def test_f32_to_f16_random_bits(oracle):
    rng = np.random.default_rng(11)
    u = rng.integers(0, 2**32, 4_000_000, dtype=np.uint64).astype(np.uint32)
    _check_f32_to_f16(oracle, u.view(np.float32))


def test_f32_to_f16_ties_and_neighbours(oracle):
    # every fp16 value, the exact midpoint to its successor, and one fp32 ulp either side
    h = np.arange(0, 0x7C00, dtype=np.uint16)
    lo = h.view(np.float16).astype(np.float64)
    hi = (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    hi[-1] = 65536.0  # midpoint above the largest finite value rounds to inf
    mid = ((lo + hi) / 2).astype(np.float32)  # exact in fp32
    cases = [lo.astype(np.float32), mid, np.nextafter(mid, np.float32(np.inf)),
             np.nextafter(mid, np.float32(-np.inf))]
    x = np.concatenate(cases)
    _check_f32_to_f16(oracle, np.concatenate([x, -x]))


def test_f32_to_f16_subnormal_and_underflow(oracle):
    e = np.arange(-30, -12)
    base = (2.0 ** e).astype(np.float32)
    fr = np.linspace(1.0, 2.0, 4097, dtype=np.float32)
    x = (base[:, None] * fr[None, :]).ravel()
    _check_f32_to_f16(oracle, np.concatenate([x, -x, [0.0, -0.0]]))
    assert oracle.f32_to_f16(np.float32([-0.0]))[0] == 0x8000
    assert oracle.f32_to_f16(np.float32([2.0 ** -25]))[0] == 0  # tie to even -> 0
    assert oracle.f32_to_f16(np.nextafter(np.float32(2.0 ** -25), np.float32(1)))[0] == 1
