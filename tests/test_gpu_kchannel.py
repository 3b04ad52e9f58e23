"""GPU parity of the paper's own INT2 key scheme (Sec. 3.2.1: keys quantised per channel over blocks of 32
tokens, tokens that do not fill a block stored at INT4) through the C ABI against the oracle: residual routing,
codes and block metadata bit-exact, every pool byte, the prefill gather bit-exact in FP16, decode attention
within the parity tolerance."""
import numpy as np
import pytest
import torch

from paper_2605_17170_amd import harness, tkv
from paper_2605_17170_amd import workloads as wl

pytestmark = pytest.mark.gpu
KC = tkv.TKV_KEYS_PER_CHANNEL


@pytest.fixture(scope="module")
def G():
    import gpu_common
    return gpu_common


@pytest.mark.parametrize("seq_lens,hkv", [([20], 1), ([64], 2), ([100], 1), ([65, 130], 3), ([200, 1, 777], 8)])
def test_append_small_ragged(G, seq_lens, hkv):
    q, K, V, seq_bits = G.random_case(11, seq_lens, hkv, hkv, f4=0.3)
    G.kc_check_append(seq_bits, K, V, hkv)[0].close()


def test_append_uniform_int2_routes_the_tail_to_int4(G):
    q, K, V, _ = G.random_case(12, [300], 2, 2)
    cache, ref = G.kc_check_append([np.full(300, 2, np.uint8)], K, V, 2)
    assert int(cache.n_tok2[0]) == 288 and int(cache.n_tok4[0]) == 12
    assert ref[0].tolist() == [2] * 288 + [4] * 12
    cache.close()


def test_append_adversarial_channels(G):
    """Constant channels, +-0, tiny and huge ranges, outlier channels, exact ties."""
    rng = np.random.default_rng(13)
    T, H = 256, 2
    x = rng.standard_normal((T, H, 128)).astype(np.float32)
    x[:, :, 0:8] *= np.float32(2.0 ** -18)
    x[:, :, 8:16] = np.float32(1.0) + x[:, :, 8:16] * np.float32(2.0 ** -9)
    x[:, :, 16:24] = np.float32(3.25)
    x[:, :, 24:32] = 0.0
    x[::2, :, 24:32] = -0.0
    x[:, :, 32:36] *= 20
    x[:, :, 40:48] *= np.float32(2.0 ** -30)
    x[:, :, 48:56] = np.clip(x[:, :, 48:56] * 16000, -65000, 65000)
    x[:, :, 56:64] = np.round(x[:, :, 56:64] * 2) / 2
    x[:, :, 64:72] = np.abs(x[:, :, 64:72])
    x[:, :, 72:80] = -np.abs(x[:, :, 72:80])
    K = wl.f32_to_bf16_bits(x)
    V = wl.f32_to_bf16_bits(np.roll(x, 77, axis=0))
    bits = np.where(np.arange(T) % 5 == 0, 4, 2).astype(np.uint8)
    G.kc_check_append([bits], K, V, H)[0].close()


def test_incremental_appends_add_blocks_to_an_open_page(G):
    """Two chunks of one sequence, each routed on its own: the first leaves an INT2 page half full (one
    block), the second adds the page's other block and must keep the first block's bits."""
    from oracle import tkv_oracle as orc
    H = 2
    q, K, V, _ = G.random_case(14, [300], H, H)
    tags = np.full(300, 2, np.uint8)
    tags[5:300:9] = 4
    chunks = [(0, 120), (120, 300)]
    desc = tkv.tkv_desc.make(H, 8, 8, int2_key_axis=KC)
    a, s = tkv.tkv_alloc_create(desc, 9), tkv.tkv_seq_create()
    pool = torch.full((tkv.tkv_pool_bytes(desc),), 0xA5, dtype=torch.uint8, device=G.DEV)
    bmap = torch.zeros(16, dtype=torch.uint8, device=G.DEV)
    status = torch.zeros(1, dtype=torch.int32, device=G.DEV)
    dK, dV = harness.bf16_tensor(K, G.DEV), harness.bf16_tensor(V, G.DEV)
    bits = np.concatenate([tkv.tkv_route_residual(tags[lo:hi]) for lo, hi in chunks])
    obits = np.concatenate([orc.route_residual(tags[lo:hi]) for lo, hi in chunks])
    assert np.array_equal(bits, obits)
    dbits = torch.from_numpy(bits).to(G.DEV)
    all_slots = []
    for lo, hi in chunks:
        slots, wp, ws = tkv.tkv_plan_append(a, s, bits[lo:hi], token_base=lo)
        all_slots.append(slots)
        tkv.tkv_quantize_append(desc, pool, bmap, dK, dV, dbits, torch.from_numpy(wp).to(G.DEV),
                                torch.from_numpy(ws).to(G.DEV), status)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    n2_first = int((bits[:120] == 2).sum())
    assert n2_first % 64 == 32, "the first chunk must leave a half-filled INT2 page"
    slots = np.concatenate(all_slots).astype(np.int64)
    Kq, Vq = orc.quantize(K, bits), orc.quantize(V, bits)
    tok = np.concatenate([orc.int2_blocks(bits[lo:hi], lo) for lo, hi in chunks])
    bs, bz = orc.quantize_k_channel(K, tok, Kq[0])
    Kq[1][bits == 2] = 0
    Kq[2][bits == 2] = 0
    o_pool = np.full(pool.numel(), 0xA5, np.uint8)
    o_map = np.zeros(16, np.uint8)
    orc.pack_pool(o_pool, o_map, H, 8, 8, slots, bits, Kq, Vq)
    orc.put_kblocks(o_pool, H, 8, slots, tok, bs, bz)
    assert np.array_equal(pool.cpu().numpy(), o_pool) and np.array_equal(bmap.cpu().numpy(), o_map)
    tkv.tkv_seq_destroy(s)
    tkv.tkv_alloc_destroy(a)


def test_incomplete_block_is_flagged_and_skipped(G):
    H = 1
    q, K, V, _ = G.random_case(15, [64], H, H)
    bits = np.full(64, 2, np.uint8)
    cache = harness.PagedCache(H, [bits], G.DEV, fill=0xA5, key_axis=KC)
    ws = cache.work_src.copy()
    ws[0, 40] = -1                      # block 1 of the page arrives with a hole
    cache.d_work_src = torch.from_numpy(ws).to(G.DEV)
    cache.append(harness.bf16_tensor(K, G.DEV), harness.bf16_tensor(V, G.DEV))
    torch.cuda.synchronize()
    assert int(cache.status.item()) == tkv.TKV_STATUS_BLOCK_PARTIAL
    from oracle import tkv_oracle as orc
    keep = np.arange(64) < 32
    Kq, Vq = orc.quantize(K[keep], bits[keep]), orc.quantize(V[keep], bits[keep])
    tok = np.arange(32, dtype=np.int64).reshape(1, 32)
    bs, bz = orc.quantize_k_channel(K[keep], tok, Kq[0])
    Kq[1][:] = 0
    Kq[2][:] = 0
    o_pool = np.full(cache.pool.numel(), 0xA5, np.uint8)
    slots = cache.slot_ids[keep].astype(np.int64)
    orc.pack_pool(o_pool, np.zeros(cache.P2 + cache.P4, np.uint8), H, cache.P2, cache.P4, slots, bits[keep], Kq, Vq)
    orc.put_kblocks(o_pool, H, cache.P2, slots, tok, bs, bz)
    assert np.array_equal(cache.pool.cpu().numpy(), o_pool)   # block 1 still holds the canary
    cache.close()


@pytest.mark.parametrize("seq_lens,hkv", [([100], 1), ([65, 130, 31], 2), ([700, 64], 8)])
def test_gather_is_bit_exact(G, seq_lens, hkv):
    from oracle import tkv_oracle as orc
    q, K, V, seq_bits = G.random_case(16, seq_lens, hkv, hkv, f4=0.3)
    cache, ref = G.kc_check_append(seq_bits, K, V, hkv)
    try:
        T = int(np.sum(seq_lens))
        Ko = torch.full((T, hkv, 128), 0x7e00, dtype=torch.int16, device=G.DEV).view(torch.float16)
        Vo = torch.full((T, hkv, 128), 0x7e00, dtype=torch.int16, device=G.DEV).view(torch.float16)
        cache.gather(Ko, Vo)
        torch.cuda.synchronize()
        assert int(cache.status.item()) == 0
        Kh, _ = G.kc_dequantized(*ref[1:])
        want_k = orc.f64_to_f16(Kh)
        want_v = orc.dequantize_f16(*ref[2])
        got_k = Ko.view(torch.int16).cpu().numpy().view(np.uint16)
        got_v = Vo.view(torch.int16).cpu().numpy().view(np.uint16)
        assert np.array_equal(got_k, want_k), "K differs at %s" % np.argwhere(got_k != want_k)[:4].tolist()
        assert np.array_equal(got_v, want_v)
    finally:
        cache.close()


@pytest.mark.parametrize("seq_lens,hq,hkv,items", [
    ([32], 1, 1, 1), ([64], 8, 1, 1), ([96], 2, 1, 2), ([100], 4, 2, 1), ([65, 130, 31], 8, 2, 3),
    ([1000, 0, 333], 16, 2, 7), ([2500], 8, 8, 9), ([4096, 777], 32, 4, 24)])
def test_decode_parity(G, seq_lens, hq, hkv, items):
    q, K, V, seq_bits = G.random_case(17, seq_lens, hq, hkv, f4=0.3)
    cache, ref = G.kc_check_append(seq_bits, K, V, hkv)
    try:
        out = G.gpu_decode(cache, q, items)
        want = G.kc_decode_ref(q, ref, seq_lens)
        G.assert_close(out, want, "per-channel keys %s" % (seq_lens,))
    finally:
        cache.close()


def test_unwritten_blocks_never_matter(G):
    """A half-filled INT2 page (one block of 32 tokens): whatever the pool held before in the other block's key
    planes (zeros, NaN patterns, fp16 numbers beyond the scale limit) neither changes an output bit nor raises
    the saturation flag (gpu_decode asserts that the status word stays 0)."""
    q, K, V, seq_bits = G.random_case(23, [96, 32], 8, 1, f4=0.0)
    outs = []
    for fill in (0x00, 0xFF, 0x7C, 0x7B):
        cache, _ = G.kc_check_append(seq_bits, K, V, 1, fill=fill)
        try:
            outs.append(G.gpu_decode(cache, q, 3))
        finally:
            cache.close()
    for o in outs[1:]:
        assert np.array_equal(outs[0], o)


def test_decode_all_int2_and_outlier_channels(G):
    """Keys with strong outlier channels, every token INT2: the case the scheme exists for."""
    q, K, V, _ = G.random_case(18, [2048], 8, 1)
    cache, ref = G.kc_check_append([np.full(2048, 2, np.uint8)], K, V, 1)
    try:
        out = G.gpu_decode(cache, q, 5)
        G.assert_close(out, G.kc_decode_ref(q, ref, [2048]), "all INT2")
    finally:
        cache.close()


def test_decode_key_scales_across_the_supported_range(G):
    """Channel ranges from 2^-12 to 2^10 (key scales up to 1023 are used exactly)."""
    rng = np.random.default_rng(19)
    T, H = 512, 1
    x = rng.standard_normal((T, H, 128)).astype(np.float32)
    x *= (np.float32(2.0) ** rng.integers(-12, 9, 128)).astype(np.float32)
    K = wl.f32_to_bf16_bits(x)
    V = wl.f32_to_bf16_bits(rng.standard_normal((T, H, 128)).astype(np.float32))
    q = wl.f32_to_bf16_bits((rng.standard_normal((1, 4, 128)) * 0.05).astype(np.float32))
    cache, ref = G.kc_check_append([np.full(T, 2, np.uint8)], K, V, H)
    try:
        assert ref[4].view(np.float16).max() > 300
        out = G.gpu_decode(cache, q, 3)
        G.assert_close(out, G.kc_decode_ref(q, ref, [T]), "key scale range")
    finally:
        cache.close()


def test_key_scale_beyond_the_limit_saturates_is_flagged_and_stays_finite(G):
    """Out of contract (per-channel key scale > 1023): the staged scale saturates, the output is wrong but
    finite and TKV_STATUS_SCALE_SATURATED is raised."""
    q, K, V, _ = G.random_case(20, [256], 8, 1)
    Ks = wl.f32_to_bf16_bits(wl.bf16_bits_to_f32(K) * np.float32(300.0))
    cache, ref = G.kc_check_append([np.full(256, 2, np.uint8)], Ks, V, 1)
    assert ref[4].view(np.float16).max() > 1023
    out = G.gpu_decode(cache, q, 3, expect_status=tkv.TKV_STATUS_SCALE_SATURATED)
    assert np.all(np.isfinite(out))
    cache.close()


def test_cfg2_full_size(G):
    """The benchmark workload with the paper's key scheme, default work-item count, every output checked."""
    w = wl.config("cfg2")
    q, K, V, _ = w.make_inputs()
    cache = harness.PagedCache(w.n_kv_heads, w.bits, G.DEV, shuffle_seed=w.seed + 1, fill=0xA5, key_axis=KC)
    try:
        g_pool, g_map = G.gpu_append(cache, K, V)
        out = G.gpu_decode(cache, q, harness.default_target_items(w.n_kv_heads))
        ref = G.kc_oracle(w.bits, K, V)
        assert np.array_equal(cache.tag_bits, ref[0])
        o_pool, o_map = G.kc_oracle_pool(cache, *ref[1:], 0xA5)
        assert np.array_equal(g_map, o_map)
        assert np.array_equal(g_pool, o_pool), "pool bytes differ at %s" % np.nonzero(g_pool != o_pool)[0][:8].tolist()
        G.assert_close(out, G.kc_decode_ref(q, ref, w.seq_lens), "cfg2 per-channel keys")
    finally:
        cache.close()
