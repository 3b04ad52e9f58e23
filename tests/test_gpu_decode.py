"""GPU parity of tkv_decode_attention (through the C ABI) against the oracle's
fp64 softmax(q K^T / sqrt(d)) V over the dequantised cache: element-wise
|gpu - ref| <= 2e-3 + 1e-2*|ref|, plus the properties that hold at any size
(split-count invariance, page-scatter invariance, exactly-representable
inputs, one-token closed form)."""
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


def _run(G, q, K, V, seq_bits, hq, hkv, targets=(1, 8), **kw):
    cache, (Kq, Vq) = G.check_append(seq_bits, K, V, hkv, **kw)
    try:
        ref = G.decode_ref(q, Kq, Vq, [b.size for b in seq_bits])
        worst = 0.0
        for t in targets:
            out = G.gpu_decode(cache, q, t)
            worst = max(worst, G.assert_close(out, ref, "target_items=%d" % t))
        return worst
    finally:
        cache.close()


@pytest.mark.parametrize("seq_lens,hq,hkv", [
    ([1], 1, 1), ([3], 4, 1), ([64], 8, 1), ([65], 8, 1), ([130, 7], 8, 2), ([200, 1, 777], 16, 2),
    ([500], 2, 1), ([129], 2, 2), ([1000, 300], 64, 8)])
def test_small_ragged(G, seq_lens, hq, hkv):
    q, K, V, seq_bits = G.random_case(11, seq_lens, hq, hkv)
    _run(G, q, K, V, seq_bits, hq, hkv, targets=(1, 5, 64))


@pytest.mark.parametrize("bits", [2, 4])
def test_uniform_width_one_stream_empty(G, bits):
    q, K, V, _ = G.random_case(12, [300, 64], 8, 2)
    _run(G, q, K, V, [np.full(300, bits, np.uint8), np.full(64, bits, np.uint8)], 8, 2, targets=(1, 7))


def test_empty_sequence_in_batch_gives_zeros(G):
    q, K, V, seq_bits = G.random_case(13, [100, 0, 50], 4, 1)
    cache, (Kq, Vq) = G.check_append(seq_bits, K, V, 1)
    out = G.gpu_decode(cache, q, 4)
    assert np.all(out[1] == 0)
    G.assert_close(out, G.decode_ref(q, Kq, Vq, [100, 0, 50]))
    cache.close()


def test_one_token_returns_its_dequantised_value(G):
    from oracle import tkv_oracle as orc
    q, K, V, _ = G.random_case(14, [1], 4, 1)
    for bits in (2, 4):
        b = [np.full(1, bits, np.uint8)]
        cache, (Kq, Vq) = G.check_append(b, K, V, 1)
        out = G.gpu_decode(cache, q, 1)
        vh = orc.dequantize(*Vq)[0, 0]
        assert np.allclose(out[0], np.broadcast_to(vh, (4, 128)), rtol=1e-6, atol=1e-6)
        cache.close()


def test_exactly_representable_cache_reproduces_unquantised_attention(G):
    """K, V on a power-of-two grid that the quantiser reproduces bit for bit:
    the kernel's output must then match plain fp64 attention on the bf16 inputs."""
    from oracle import tkv_oracle as orc
    rng = np.random.default_rng(15)
    T, hq, hkv = 500, 8, 2
    bits = rng.choice([2, 4], T).astype(np.uint8)
    vals = np.empty((2, T, hkv, 128))
    for b, (z, s) in ((2, (-1.0, 0.5)), (4, (-2.0, 0.25))):
        n = int((bits == b).sum())
        c = rng.integers(0, 2 ** b, (2, n, hkv, 4, 32))
        c[..., 0] = 0
        c[..., 1] = 2 ** b - 1
        vals[:, bits == b] = (z + s * rng.permuted(c, axis=-1)).reshape(2, n, hkv, 128)
    K, V = wl.f32_to_bf16_bits(vals[0].astype(np.float32)), wl.f32_to_bf16_bits(vals[1].astype(np.float32))
    q = wl.make_q(np.random.SeedSequence(16), 1, hq)
    cache, (Kq, Vq) = G.check_append([bits], K, V, hkv)
    assert np.array_equal(orc.dequantize(*Kq), vals[0])
    ref = orc.attention_f64(wl.bf16_bits_to_f32(q).astype(np.float64), vals[0], vals[1], [0, T], G.SM)
    G.assert_close(G.gpu_decode(cache, q, 6), ref)
    cache.close()


def test_split_count_and_page_scatter_invariance(G):
    q, K, V, seq_bits = G.random_case(17, [3000, 1500], 8, 1)
    outs = []
    for seed, factor in ((0, 1.0), (5, 3.0)):
        cache, (Kq, Vq) = G.check_append(seq_bits, K, V, 1, shuffle_seed=seed, pool_factor=factor)
        for t in (1, 2, 7, 64, 500):
            outs.append(G.gpu_decode(cache, q, t))
        cache.close()
    ref = G.decode_ref(q, Kq, Vq, [3000, 1500])
    for o in outs:
        G.assert_close(o, ref)
        # different split counts / page placements only reorder fp32 sums: 10x inside the parity tolerance
        assert np.allclose(o, outs[0], rtol=1e-3, atol=2e-4)


def test_hundreds_of_items_per_sequence(G):
    """One long sequence on one kv head cut into one item per page: the cross-split reduction then runs in its
    wide shape (channel slices, 32 item groups per slice); same result as with few items."""
    q, K, V, seq_bits = G.random_case(27, [12800], 4, 1)
    cache, (Kq, Vq) = G.check_append(seq_bits, K, V, 1)
    try:
        ref = G.decode_ref(q, Kq, Vq, [12800])
        for target in (1000, 3):
            out = G.gpu_decode(cache, q, target)
            n_items = cache._plan[2].shape[0]
            assert (n_items > 128) == (target == 1000)
            G.assert_close(out, ref, "target_items=%d (%d items)" % (target, n_items))
    finally:
        cache.close()


def test_workspace_and_output_are_written_inside_their_bounds(G):
    """Guard words behind the workspace (sized by tkv_decode_workspace_bytes) and around `out` keep their canary."""
    q, K, V, seq_bits = G.random_case(28, [700, 130], 8, 2)
    cache, (Kq, Vq) = G.check_append(seq_bits, K, V, 2)
    try:
        items, _ = cache.plan_decode(9)
        need = tkv.tkv_decode_workspace_bytes(cache.desc, items.shape[0], 8)
        guard = 4096
        ws = torch.full((need + guard,), 0x5A, dtype=torch.uint8, device=G.DEV)
        obuf = torch.full((guard + 2 * 8 * 128 * 4 + guard,), 0x5A, dtype=torch.uint8, device=G.DEV)
        out = obuf[guard:guard + 2 * 8 * 128 * 4].view(torch.float32).view(2, 8, 128)
        cache.decode(harness.bf16_tensor(q, G.DEV), out=out, workspace=ws[:need])
        torch.cuda.synchronize()
        assert int(cache.status.item()) == 0
        assert bool((ws[need:] == 0x5A).all()), "write behind the workspace"
        assert bool((obuf[:guard] == 0x5A).all()) and bool((obuf[-guard:] == 0x5A).all()), "write outside out"
        G.assert_close(out.cpu().numpy(), G.decode_ref(q, Kq, Vq, [700, 130]), "guarded buffers")
    finally:
        cache.close()


def test_decode_on_oracle_packed_pool(G):
    """Isolates decode from append: the pool bytes come from the oracle's codec."""
    q, K, V, seq_bits = G.random_case(18, [700, 90], 8, 2)
    from oracle import tkv_oracle as orc
    cache = harness.PagedCache(2, seq_bits, G.DEV, pool_factor=2.0, shuffle_seed=4, fill=0xA5)
    Kq, Vq = orc.quantize(K, cache.tag_bits), orc.quantize(V, cache.tag_bits)
    pool, bmap = G.oracle_pool(cache, Kq, Vq, 0xA5)
    cache.pool.copy_(torch.from_numpy(pool).to(G.DEV))
    cache.bit_map.copy_(torch.from_numpy(bmap).to(G.DEV))
    G.assert_close(G.gpu_decode(cache, q, 9), G.decode_ref(q, Kq, Vq, [700, 90]))
    cache.close()


def test_unwritten_slots_never_matter(G):
    """Same tokens, pool pre-filled with different garbage (0x00, 0xFF and 0x7C = NaN
    patterns in the metadata planes, 0x7B = fp16 numbers beyond the V scale limit):
    identical output bits, and no status bit (gpu_decode asserts that)."""
    q, K, V, seq_bits = G.random_case(19, [100, 37], 8, 1)
    outs = []
    for fill in (0x00, 0xFF, 0x7C, 0x7B):
        cache, _ = G.check_append(seq_bits, K, V, 1, fill=fill)
        outs.append(G.gpu_decode(cache, q, 3))
        cache.close()
    assert all(np.array_equal(outs[0], o) for o in outs[1:])


def test_bitmap_mismatch_is_flagged(G):
    q, K, V, seq_bits = G.random_case(20, [128], 4, 1)
    cache, _ = G.check_append(seq_bits, K, V, 1)
    cache.bit_map.zero_()
    cache.plan_decode(2)
    cache.decode(harness.bf16_tensor(q, G.DEV))
    torch.cuda.synchronize()
    assert int(cache.status.item()) & tkv.TKV_STATUS_BITMAP_MISMATCH
    cache.close()


def test_large_q_and_peaked_softmax(G):
    """q scaled by 8 (logit standard deviation ~30): softmax close to one-hot."""
    q, K, V, seq_bits = G.random_case(21, [2000], 8, 1)
    qf = wl.bf16_bits_to_f32(q) * np.float32(8.0)
    _run(G, wl.f32_to_bf16_bits(qf), K, V, seq_bits, 8, 1, targets=(1, 16))
    qf = wl.bf16_bits_to_f32(q) * np.float32(2.0 ** -12)
    _run(G, wl.f32_to_bf16_bits(qf), K, V, seq_bits, 8, 1, targets=(4,))


def test_v_magnitudes_across_the_supported_range(G):
    """The kernel multiplies the softmax weights by the V scale in fp16: V scaled by 4 (INT2 scales of
    the outlier groups ~200, close to the documented limit of 255) and by 2^-10 (staged scales in the
    fp16 subnormal range) must still meet the tolerance."""
    q, K, V, seq_bits = G.random_case(22, [700, 100], 8, 1)
    for f in (4.0, 2.0 ** -10):
        Vs = wl.f32_to_bf16_bits(wl.bf16_bits_to_f32(V) * np.float32(f))
        _run(G, q, K, Vs, seq_bits, 8, 1, targets=(1, 9))


def test_v_scale_beyond_the_limit_saturates_is_flagged_and_stays_finite(G):
    """Out of contract (V scale > 255): the staged scale saturates, the output is wrong but finite and
    TKV_STATUS_SCALE_SATURATED is raised; a cache just inside the limit raises nothing and is in tolerance."""
    q, K, V, seq_bits = G.random_case(23, [300], 8, 1)
    Vs = wl.f32_to_bf16_bits(wl.bf16_bits_to_f32(V) * np.float32(64.0))
    cache, _ = G.check_append(seq_bits, K, Vs, 1)
    out = G.gpu_decode(cache, q, 3, expect_status=tkv.TKV_STATUS_SCALE_SATURATED)
    assert np.all(np.isfinite(out))
    cache.close()
    Vs = wl.f32_to_bf16_bits(wl.bf16_bits_to_f32(V) * np.float32(4.0))      # INT2 scales of the x20 channels reach ~200
    cache, (Kq, Vq) = G.check_append(seq_bits, K, Vs, 1)
    assert Vq[1].view(np.float16).max() > 100
    G.assert_close(G.gpu_decode(cache, q, 3), G.decode_ref(q, Kq, Vq, [300]), "V scales up to %.0f" % Vq[1].view(np.float16).max())
    cache.close()


def test_item_naming_a_sequence_outside_the_batch_is_flagged_and_contributes_nothing(G):
    q, K, V, seq_bits = G.random_case(24, [400, 200], 8, 2)
    cache, (Kq, Vq) = G.check_append(seq_bits, K, V, 2)
    try:
        ref = G.decode_ref(q, Kq, Vq, [400, 200])
        items, sip = cache.plan_decode(6)
        bad = items.copy()
        k = int(np.nonzero(items[:, 3] == sip[1] - 1)[0][0])   # the last item of sequence 0 is replaced by a malformed one
        lost = bad[k].copy()
        bad[k, 0] = 7
        cache._plan = (torch.from_numpy(bad).to(G.DEV), cache._plan[1], bad, sip)
        ws = cache.workspace(8)
        ws.view(torch.float32).fill_(float("nan"))   # whatever an earlier call left there must not reach the output
        out = cache.decode(harness.bf16_tensor(q, G.DEV), workspace=ws)
        torch.cuda.synchronize()
        assert int(cache.status.item()) == tkv.TKV_STATUS_BAD_ITEM
        out = out.cpu().numpy()
        assert np.all(np.isfinite(out))
        G.assert_close(out[1:], ref[1:], "the untouched sequence")
        # sequence 0 is attention over the pages of its remaining items: compare with the oracle on those tokens
        from oracle import tkv_oracle as orc
        keep = np.ones(400, bool)
        slots = cache.slot_ids[:400].astype(np.int64)
        pages0 = cache.page_ids[cache.page_indptr[0]:cache.page_indptr[1]]
        dropped = set(int(p) for p in pages0[lost[1]:lost[2]])
        for t in range(400):
            keep[t] = int(slots[t] // 64) not in dropped
        sel = np.nonzero(keep)[0]
        Kq0 = tuple(a[sel] for a in Kq)
        Vq0 = tuple(a[sel] for a in Vq)
        ref0 = G.decode_ref(q[:1], Kq0, Vq0, [sel.size])
        G.assert_close(out[:1], ref0, "sequence 0 without the malformed item's pages")
    finally:
        cache.close()


def test_item_with_a_partial_slot_outside_the_workspace_is_flagged_and_writes_nothing(G):
    """The partial of such an item cannot be stored: the status bit is raised, nothing outside the workspace is
    touched (guard words behind it), and the sequences whose slots were all written are unaffected."""
    q, K, V, seq_bits = G.random_case(25, [400, 200], 8, 2)
    cache, (Kq, Vq) = G.check_append(seq_bits, K, V, 2)
    try:
        ref = G.decode_ref(q, Kq, Vq, [400, 200])
        items, sip = cache.plan_decode(6)
        for wrong in (items.shape[0], items.shape[0] + 1000, -1):
            bad = items.copy()
            k = int(np.nonzero(items[:, 3] == sip[1] - 1)[0][0])   # an item of sequence 0
            bad[k, 3] = wrong
            cache._plan = (torch.from_numpy(bad).to(G.DEV), cache._plan[1], bad, sip)
            need = tkv.tkv_decode_workspace_bytes(cache.desc, items.shape[0], 8)
            buf = torch.full((need + 4096,), 0x5A, dtype=torch.uint8, device=G.DEV)
            cache.status.zero_()
            out = cache.decode(harness.bf16_tensor(q, G.DEV), workspace=buf[:need])
            torch.cuda.synchronize()
            assert int(cache.status.item()) == tkv.TKV_STATUS_BAD_ITEM
            assert bool((buf[need:] == 0x5A).all()), "bytes behind the workspace were written"
            G.assert_close(out.cpu().numpy()[1:], ref[1:], "the sequence whose slots were all written")
    finally:
        cache.close()


def test_many_short_sequences_more_items_than_fit_the_device(G):
    """700 sequences of 1..200 tokens (some empty) on 8 kv heads: more (item, head) workgroups than the device
    holds at once whatever the target, so late workgroups start when early ones end; one item per sequence."""
    rng = np.random.default_rng(31)
    seq_lens = rng.integers(1, 200, 700).tolist()
    for k in (5, 333, 699):
        seq_lens[k] = 0
    q, K, V, seq_bits = G.random_case(31, seq_lens, 8, 8)
    _run(G, q, K, V, seq_bits, 8, 8, targets=(1, 384))


def test_cfg1(G):
    w = wl.config("cfg1")
    q, K, V, _ = w.make_inputs()
    _run(G, q, K, V, w.bits, w.n_q_heads, w.n_kv_heads, targets=(1, 8, 32))


@pytest.mark.parametrize("name,scale", [("cfg2", 0.125), ("cfg3", 0.1), ("cfg5", 0.05)])
def test_scaled_configs(G, name, scale):
    w = wl.config(name, scale)
    q, K, V, _ = w.make_inputs()
    factor = 4.0 if name == "cfg3" else 1.0
    _run(G, q, K, V, w.bits, w.n_q_heads, w.n_kv_heads,
         targets=(harness.default_target_items(w.n_kv_heads),), pool_factor=factor)
