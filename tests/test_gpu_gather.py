"""GPU parity of tkv_gather_dequant (prefill gather, through the C ABI) against the oracle: every FP16 value
bit-exact (nearest-even of the exact code * scale + zero); rows that no slot names keep their canary."""
import numpy as np
import pytest
import torch

from paper_2605_17170_amd import harness, tkv
from paper_2605_17170_amd import workloads as wl

pytestmark = pytest.mark.gpu

CANARY = 0x7e11   # an fp16 NaN pattern that no dequantised value produces


@pytest.fixture(scope="module")
def G():
    import gpu_common
    return gpu_common


def _gather(G, cache, n_tokens, hkv):
    Ko = torch.full((n_tokens, hkv, 128), CANARY, dtype=torch.int16, device=G.DEV).view(torch.float16)
    Vo = torch.full((n_tokens, hkv, 128), CANARY, dtype=torch.int16, device=G.DEV).view(torch.float16)
    cache.gather(Ko, Vo)
    torch.cuda.synchronize()
    assert int(cache.status.item()) == 0
    return Ko.view(torch.int16).cpu().numpy().view(np.uint16), Vo.view(torch.int16).cpu().numpy().view(np.uint16)


def _check(G, seq_bits, K, V, hkv, **kw):
    from oracle import tkv_oracle as orc
    cache, (Kq, Vq) = G.check_append(seq_bits, K, V, hkv, **kw)
    try:
        gK, gV = _gather(G, cache, K.shape[0], hkv)
        for name, got, q in (("K", gK, Kq), ("V", gV, Vq)):
            want = orc.dequantize_f16(*q)
            bad = np.argwhere(got != want)
            assert bad.size == 0, "%s differs at %s: gpu %04x oracle %04x" % (
                name, bad[0].tolist(), got[tuple(bad[0])], want[tuple(bad[0])])
    finally:
        cache.close()


@pytest.mark.parametrize("seq_lens,hkv", [([1], 1), ([5], 2), ([64], 1), ([65, 130], 3), ([200, 1, 777], 8)])
def test_small_ragged(G, seq_lens, hkv):
    q, K, V, seq_bits = G.random_case(41, seq_lens, hkv, hkv)
    _check(G, seq_bits, K, V, hkv)


@pytest.mark.parametrize("bits", [2, 4])
def test_uniform_width(G, bits):
    q, K, V, _ = G.random_case(42, [300], 2, 2)
    _check(G, [np.full(300, bits, np.uint8)], K, V, 2)


def test_wide_value_range(G):
    """Scales from tiny to large and large negative zeros: the single rounding matters most here."""
    rng = np.random.default_rng(43)
    T, hkv = 500, 2
    x = rng.standard_normal((2, T, hkv, 128)) * 10.0 ** rng.integers(-4, 3, (2, T, hkv, 4, 1)).repeat(32, axis=-1).reshape(2, T, hkv, 128)
    x += 10.0 ** rng.integers(-2, 3, (2, T, hkv, 1)) * rng.choice([-1.0, 1.0], (2, T, hkv, 1))
    K, V = wl.f32_to_bf16_bits(x[0].astype(np.float32)), wl.f32_to_bf16_bits(x[1].astype(np.float32))
    bits = rng.choice([2, 4], T).astype(np.uint8)
    _check(G, [bits], K, V, hkv)


def test_unlisted_rows_and_slots_are_untouched(G):
    """Only half of the pages are listed and some slots are masked with -1: every other row keeps the canary."""
    from oracle import tkv_oracle as orc
    q, K, V, seq_bits = G.random_case(44, [400, 90], 2, 2)
    cache, (Kq, Vq) = G.check_append(seq_bits, K, V, 2)
    try:
        T = K.shape[0]
        keep = np.arange(cache.work_pages.size) % 2 == 0
        wp = cache.work_pages[keep].copy()
        wd = cache.work_src[keep].copy()
        wd[:, ::5] = -1
        Ko = torch.full((T, 2, 128), CANARY, dtype=torch.int16, device=G.DEV).view(torch.float16)
        Vo = torch.full((T, 2, 128), CANARY, dtype=torch.int16, device=G.DEV).view(torch.float16)
        tkv.tkv_gather_dequant(cache.desc, cache.pool, cache.bit_map, torch.from_numpy(wp).to(G.DEV),
                               torch.from_numpy(wd).to(G.DEV), Ko, Vo, cache.status)
        torch.cuda.synchronize()
        assert int(cache.status.item()) == 0
        gK = Ko.view(torch.int16).cpu().numpy().view(np.uint16)
        gV = Vo.view(torch.int16).cpu().numpy().view(np.uint16)
        listed = np.zeros(T, bool)
        listed[wd[wd >= 0]] = True
        assert listed.any() and not listed.all()
        wantK, wantV = orc.dequantize_f16(*Kq), orc.dequantize_f16(*Vq)
        assert np.array_equal(gK[listed], wantK[listed]) and np.array_equal(gV[listed], wantV[listed])
        assert np.all(gK[~listed] == CANARY) and np.all(gV[~listed] == CANARY)
    finally:
        cache.close()


def test_errors_are_flagged_not_read(G):
    q, K, V, seq_bits = G.random_case(45, [130], 1, 1)
    cache, _ = G.check_append(seq_bits, K, V, 1, pool_factor=3.0)
    try:
        T = K.shape[0]
        Ko = torch.full((T, 1, 128), CANARY, dtype=torch.int16, device=G.DEV).view(torch.float16)
        Vo = Ko.clone()
        used = set(cache.work_pages.tolist())
        unused = next(p for p in range(cache.P2 + cache.P4) if p not in used)   # never written: bit_map 0
        wp = np.array([unused, cache.P2 + cache.P4 + 7, cache.work_pages[0]], np.int32)
        wd = np.full((3, 64), -1, np.int32)
        wd[0, 0] = 0
        wd[1, 0] = 1
        wd[2, 0] = T + 5          # beyond the output
        tkv.tkv_gather_dequant(cache.desc, cache.pool, cache.bit_map, torch.from_numpy(wp).to(G.DEV),
                               torch.from_numpy(wd).to(G.DEV), Ko, Vo, cache.status)
        torch.cuda.synchronize()
        st = int(cache.status.item())
        assert st == tkv.TKV_STATUS_BITMAP_MISMATCH | tkv.TKV_STATUS_PAGE_RANGE | tkv.TKV_STATUS_DST_RANGE
        assert bool((Ko.view(torch.int16) == CANARY).all()) and bool((Vo.view(torch.int16) == CANARY).all())
    finally:
        cache.close()


def test_cfg4_full(G):
    """BASELINE config 4 at full size: 65 536 tokens x 8 heads, every value compared."""
    w = wl.config("cfg4")
    q, K, V, _ = w.make_inputs()
    _check(G, w.bits, K, V, w.n_kv_heads, pool_factor=1.0)
