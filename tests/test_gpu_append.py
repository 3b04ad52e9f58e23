"""GPU parity of tkv_quantize_append (through the C ABI) against the oracle:
codes, fp16 scales and fp16 zero-points bit-exact, and every byte of the pool
equal to the oracle-packed pool (a 0xA5 canary fill shows stray writes)."""
import numpy as np
import pytest
import torch

from paper_2605_17170_amd import harness, tkv
from paper_2605_17170_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import gpu_common
    return gpu_common


@pytest.mark.parametrize("seq_lens,hkv", [([1], 1), ([5], 2), ([64], 1), ([65, 130], 3), ([200, 1, 777], 8)])
def test_small_ragged(G, seq_lens, hkv):
    q, K, V, seq_bits = G.random_case(1, seq_lens, hkv, hkv)
    G.check_append(seq_bits, K, V, hkv)[0].close()


@pytest.mark.parametrize("bits", [2, 4])
def test_uniform_width(G, bits):
    q, K, V, _ = G.random_case(2, [300], 2, 2)
    G.check_append([np.full(300, bits, np.uint8)], K, V, 2)[0].close()


def test_empty_append_is_a_noop(G):
    cache = harness.PagedCache(2, [np.zeros(0, np.uint8)], G.DEV, fill=0xA5)
    K = torch.empty((0, 2, 128), dtype=torch.bfloat16, device=G.DEV)
    cache.append(K, K)
    torch.cuda.synchronize()
    assert bool((cache.pool == 0xA5).all()) and int(cache.bit_map.sum()) == 0
    cache.close()


def test_adversarial_values(G):
    """Tiny ranges, constant groups, +-0, large outliers, values near fp16's
    subnormal range and at the top of the allowed magnitude."""
    rng = np.random.default_rng(7)
    T, H = 256, 2
    x = rng.standard_normal((T, H, 4, 32)).astype(np.float32)
    x[0:16] *= np.float32(2.0 ** -18)                      # scale in fp16's subnormal range
    x[16:32] = np.float32(1.0) + x[16:32] * np.float32(2.0 ** -9)    # tiny range on an offset
    x[32:48] = np.float32(3.25)                            # constant groups
    x[48:64] = 0.0
    x[48:64, :, :, ::2] = -0.0
    x[64:80, :, :, 5] *= 20                                # one outlier channel per group
    x[80:96] *= np.float32(2.0 ** -30)                     # scale underflows to zero
    x[96:112] *= 16000                                     # large magnitudes (|x| < 65504)
    x[96:112] = np.clip(x[96:112], -65000, 65000)
    x[112:128] = np.round(x[112:128] * 2) / 2              # exact ties for the rounding rule
    x[128:144] = np.abs(x[128:144])                        # minimum > 0
    x[144:160] = -np.abs(x[144:160])                       # maximum < 0
    K = wl.f32_to_bf16_bits(x.reshape(T, H, 128))
    V = wl.f32_to_bf16_bits(np.roll(x, 77, axis=0).reshape(T, H, 128))
    bits = np.tile(np.uint8([2, 4]), T // 2)
    G.check_append([bits], K, V, H)[0].close()


def test_incremental_appends_fill_partial_pages(G):
    """Three calls on one sequence: later calls add tokens to partly filled
    pages of both widths and must keep the earlier tokens' bits."""
    from oracle import tkv_oracle as orc
    H = 2
    q, K, V, seq_bits = G.random_case(3, [333], H, H)
    bits = seq_bits[0]
    desc = tkv.tkv_desc.make(H, 8, 8)
    a, s = tkv.tkv_alloc_create(desc, 9), tkv.tkv_seq_create()
    pool = torch.full((tkv.tkv_pool_bytes(desc),), 0xA5, dtype=torch.uint8, device=G.DEV)
    bmap = torch.zeros(16, dtype=torch.uint8, device=G.DEV)
    status = torch.zeros(1, dtype=torch.int32, device=G.DEV)
    dK, dV = harness.bf16_tensor(K, G.DEV), harness.bf16_tensor(V, G.DEV)
    dbits = torch.from_numpy(bits).to(G.DEV)
    all_slots = []
    for lo, hi in [(0, 100), (100, 101), (101, 333)]:
        slots, wp, ws = tkv.tkv_plan_append(a, s, bits[lo:hi], token_base=lo)
        all_slots.append(slots)
        tkv.tkv_quantize_append(desc, pool, bmap, dK, dV, dbits, torch.from_numpy(wp).to(G.DEV),
                                torch.from_numpy(ws).to(G.DEV), status)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    slots = np.concatenate(all_slots).astype(np.int64)
    Kq, Vq = orc.quantize(K, bits), orc.quantize(V, bits)
    o_pool = np.full(pool.numel(), 0xA5, np.uint8)
    o_map = np.zeros(16, np.uint8)
    orc.pack_pool(o_pool, o_map, H, 8, 8, slots, bits, Kq, Vq)
    assert np.array_equal(pool.cpu().numpy(), o_pool) and np.array_equal(bmap.cpu().numpy(), o_map)
    tkv.tkv_seq_destroy(s)
    tkv.tkv_alloc_destroy(a)


def test_tag_mismatch_is_flagged_and_skipped(G):
    H = 1
    q, K, V, _ = G.random_case(4, [64], H, H)
    bits = np.full(64, 2, np.uint8)
    cache = harness.PagedCache(H, [bits], G.DEV, fill=0xA5)
    wrong = bits.copy()
    wrong[10] = 4                       # device-side tag disagrees with the page's pool
    cache.d_tag_bits = torch.from_numpy(wrong).to(G.DEV)
    cache.append(harness.bf16_tensor(K, G.DEV), harness.bf16_tensor(V, G.DEV))
    torch.cuda.synchronize()
    assert int(cache.status.item()) == tkv.TKV_STATUS_TAG_MISMATCH
    from oracle import tkv_oracle as orc
    keep = np.arange(64) != 10
    Kq, Vq = orc.quantize(K[keep], bits[keep]), orc.quantize(V[keep], bits[keep])
    o_pool = np.full(cache.pool.numel(), 0xA5, np.uint8)
    orc.pack_pool(o_pool, np.zeros(cache.P2 + cache.P4, np.uint8), H, cache.P2, cache.P4,
                  cache.slot_ids[keep].astype(np.int64), bits[keep], Kq, Vq)
    assert np.array_equal(cache.pool.cpu().numpy(), o_pool)   # slot 10 still holds the canary
    cache.close()


def test_cfg1_and_scaled_cfg4(G):
    for name, scale in (("cfg1", 1.0), ("cfg4", 0.125)):
        w = wl.config(name, scale)
        q, K, V, _ = w.make_inputs()
        G.check_append(w.bits, K, V, w.n_kv_heads)[0].close()


def test_cfg4_full_size(G):
    """65536 tokens x 8 kv heads in one call, randomly allocated pages; every pool byte checked."""
    w = wl.config("cfg4")
    q, K, V, _ = w.make_inputs()
    cache, _ = G.check_append(w.bits, K, V, w.n_kv_heads, pool_factor=1.25)
    assert cache.work_pages.size == 1024
    cache.close()


@pytest.mark.parametrize("axis", [tkv.TKV_KEYS_PER_TOKEN, tkv.TKV_KEYS_PER_CHANNEL])
def test_random_bf16_bit_patterns(G, axis):
    """Values drawn as raw bf16 bit patterns (every finite exponent up to 2^15, both signs, subnormals, +-0) mixed
    with narrow-range groups: ties, clamping on both sides, scales that overflow to the top of fp16 or flush to 0."""
    rng = np.random.default_rng(41)
    T, H = 2048, 4
    def draw():
        b = rng.integers(0, 1 << 16, (T, H, 128), dtype=np.uint16)
        exp = (b >> 7) & 0xff
        b = np.where(exp > 141, (b & 0x807f) | (np.uint16(141) << 7), b).astype(np.uint16)   # |x| < 2^15
        narrow = rng.random((T, H, 4, 1)) < 0.5                                              # half of the groups: one binade
        base = rng.integers(100, 140, (T, H, 4, 1)).astype(np.uint16)
        nb = ((b.reshape(T, H, 4, 32) & 0x807f) | (base << 7)).astype(np.uint16)
        return np.where(narrow, nb, b.reshape(T, H, 4, 32)).reshape(T, H, 128).astype(np.uint16)
    K, V = draw(), draw()
    bits = rng.choice([2, 4], T).astype(np.uint8)
    if axis == tkv.TKV_KEYS_PER_CHANNEL:
        G.kc_check_append([bits], K, V, H)[0].close()
    else:
        G.check_append([bits], K, V, H)[0].close()
