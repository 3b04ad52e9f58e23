"""Pins for the oracle's per-channel INT2 keys (paper Sec. 3.2.1: INT2 keys are quantised per channel over a
block of G = 32 tokens; tokens that do not fill a block take the INT4 per-token path).

Nothing here re-types the oracle's code: the pins are a hand-worked block (tests/golden/
kchannel_worked_block.txt), numpy's own reductions and fp16 casts along the token axis, an exact-arithmetic
nearest-code search, the already pinned per-token quantiser on the transposed block (axis handling), the
outlier-isolation property that motivates the scheme, hand-derived positions of the metadata layout, and
closed cases of the residual policy."""
import os
from fractions import Fraction

import numpy as np
import pytest

from paper_2605_17170_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden", "kchannel_worked_block.txt")


def _load_block():
    chans, cur = [], None
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line.startswith("channel "):
            parts = line.split()
            cur = {"name": parts[1]}
            for p in parts[2:]:
                k, v = p.split("=")
                cur[k] = int(v, 16)
            chans.append(cur)
        elif line.startswith("x:"):
            cur["x"] = [float(v) for v in line[2:].split()]
        elif line.startswith("c:"):
            cur["c"] = [int(v) for v in line[2:].split()]
    return chans


def _quant_block(oracle, xb, tok=None, T=None):
    """xb bf16 bits [T,H,D]; one or more blocks given by tok [nb,32]."""
    T = xb.shape[0]
    tok = np.arange(T, dtype=np.int64).reshape(-1, 32) if tok is None else tok
    codes = np.full(xb.shape, 255, np.uint8)
    bs, bz = oracle.quantize_k_channel(xb, tok, codes)
    return codes, bs, bz


def test_worked_block(oracle):
    chans = _load_block()
    assert [c["name"] for c in chans] == ["A", "B", "C", "D"]
    D = 128
    x = np.zeros((32, 1, D), np.float32)
    for i, ch in enumerate(chans):
        assert len(ch["x"]) == 32 and len(ch["c"]) == 32
        x[:, 0, 40 * i + 3] = ch["x"]          # scattered over the head so a channel/group mix-up shows
    xb = wl.f32_to_bf16_bits(x)
    assert np.array_equal(wl.bf16_bits_to_f32(xb), x), "fixture values must be bf16-exact"
    codes, bs, bz = _quant_block(oracle, xb)
    for i, ch in enumerate(chans):
        c = 40 * i + 3
        assert bs[0, 0, c] == ch["scale"] and bz[0, 0, c] == ch["zero"], ch["name"]
        assert codes[:, 0, c].tolist() == ch["c"], ch["name"]
    # the untouched channels are constant zero: scale 0, zero 0, codes 0
    rest = np.ones(D, bool)
    rest[[40 * i + 3 for i in range(4)]] = False
    assert not bs[0, 0, rest].any() and not bz[0, 0, rest].any() and not codes[:, 0, rest].any()


def _random_tokens(rng, T, H, kind):
    x = rng.standard_normal((T, H, 128)).astype(np.float32)
    if kind == "outlier":
        x[:, :, [5, 37, 90, 127]] *= 20          # outlier CHANNELS, as in keys
    elif kind == "shifted":
        x = x * np.float32(0.01) + rng.uniform(-50, 50, (1, H, 128)).astype(np.float32)
    elif kind == "halves":
        x = np.round(x * 4) / 4
    return wl.f32_to_bf16_bits(x)


@pytest.mark.parametrize("kind", ["normal", "outlier", "shifted", "halves"])
def test_scale_zero_are_numpy_reductions_over_the_token_axis(oracle, kind):
    rng = np.random.default_rng(400)
    T, H = 96, 3
    xb = _random_tokens(rng, T, H, kind)
    tok = rng.permutation(T).astype(np.int64).reshape(3, 32)     # blocks of scattered rows
    codes, bs, bz = _quant_block(oracle, xb, tok)
    x = wl.bf16_bits_to_f32(xb)
    for b in range(3):
        blk = x[tok[b]]                                          # [32,H,D]
        mn, mx = blk.min(axis=0), blk.max(axis=0)
        want_s = (np.float32(mx - mn) / np.float32(3)).astype(np.float16).view(np.uint16)
        want_z = (mn + np.float32(0)).astype(np.float16).view(np.uint16)
        assert np.array_equal(bs[b], want_s) and np.array_equal(bz[b], want_z)
    assert codes.max() <= 3


@pytest.mark.parametrize("kind", ["normal", "outlier", "halves"])
def test_codes_are_nearest_levels_of_the_channel(oracle, kind):
    """Exact arithmetic: the code is the level zero_c + k * scale_c nearest to x (near-ties skipped)."""
    rng = np.random.default_rng(401)
    xb = _random_tokens(rng, 32, 1, kind)
    codes, bs, bz = _quant_block(oracle, xb)
    x = wl.bf16_bits_to_f32(xb)
    checked = 0
    for c in range(128):
        sf = Fraction(float(bs[0, 0, c:c + 1].view(np.float16)[0]))
        zf = Fraction(float(bz[0, 0, c:c + 1].view(np.float16)[0]))
        if sf == 0:
            assert not codes[:, 0, c].any()
            continue
        for t in range(32):
            v = (Fraction(float(x[t, 0, c])) - zf) / sf
            fl = v.numerator // v.denominator
            frac = v - fl
            if abs(frac - Fraction(1, 2)) < Fraction(1, 4096):
                continue
            k = min(max(fl + (1 if frac > Fraction(1, 2) else 0), 0), 3)
            assert codes[t, 0, c] == k
            checked += 1
    assert checked > 3500


def test_equals_the_per_token_quantiser_on_the_transposed_block(oracle):
    """A channel's 32 token values, laid out as the 32 channels of one group of a synthetic token, must give
    the same codes / scale / zero through the per-token path (pinned in test_oracle_quantizer.py)."""
    rng = np.random.default_rng(402)
    H = 2
    xb = _random_tokens(rng, 64, H, "outlier")
    tok = np.stack([np.arange(0, 64, 2), np.arange(1, 64, 2)]).astype(np.int64)   # interleaved blocks
    codes, bs, bz = _quant_block(oracle, xb, tok)
    for b in range(2):
        xt = np.ascontiguousarray(xb[tok[b]].transpose(2, 1, 0))      # [D "tokens", H, 32 "channels"]
        c2, s2, z2 = oracle.quantize(xt, np.full(128, 2, np.uint8), G=32)
        assert np.array_equal(codes[tok[b]].transpose(2, 1, 0), c2)
        assert np.array_equal(bs[b].T, s2[..., 0]) and np.array_equal(bz[b].T, z2[..., 0])


def test_outlier_channels_do_not_touch_their_neighbours(oracle):
    """The reason for the scheme (Sec. 3.2.1): scaling one channel by 20 changes that channel's scale and
    nothing else, whereas under per-token groups it changes the codes of its 31 group neighbours."""
    rng = np.random.default_rng(403)
    xb = _random_tokens(rng, 32, 1, "normal")
    y = wl.f32_to_bf16_bits(wl.bf16_bits_to_f32(xb) * np.where(np.arange(128) == 37, np.float32(16), np.float32(1)))
    ca, sa, za = _quant_block(oracle, xb)
    cb, sb, zb = _quant_block(oracle, y)
    other = np.arange(128) != 37
    assert np.array_equal(ca[:, :, other], cb[:, :, other])
    assert np.array_equal(sa[..., other], sb[..., other]) and np.array_equal(za[..., other], zb[..., other])
    # a power-of-two factor scales the channel's grid exactly: same codes, scale and zero times 16
    assert np.array_equal(ca[:, :, 37], cb[:, :, 37])
    assert sb[0, 0, 37:38].view(np.float16)[0] == 16 * sa[0, 0, 37:38].view(np.float16)[0]
    # per-token groups: the same change wrecks the neighbours of channel 37 in every token
    pa = oracle.quantize(xb, np.full(32, 2, np.uint8))[0]
    pb = oracle.quantize(y, np.full(32, 2, np.uint8))[0]
    nb = (np.arange(128) // 32 == 1) & other
    assert (pa[:, :, nb] != pb[:, :, nb]).mean() > 0.3


def test_round_trip_and_dequantisation(oracle):
    """x_hat = code * scale_c + zero_c: exact on grids that the codes can represent, within half a step
    (plus the fp16 shortfall of the scale at the top code) elsewhere."""
    rng = np.random.default_rng(404)
    # exactly representable: channel c holds zero_c + k * 2^e_c, k in 0..3, both extremes present
    e = rng.integers(-6, 5, 128)
    z = rng.integers(-16, 17, 128) * np.float32(2.0) ** e          # x = (m + k) 2^e: bf16- and fp16-exact
    k = rng.integers(0, 4, (32, 1, 128))
    k[0], k[1] = 0, 3
    x = (z + k * np.float32(2.0) ** e).astype(np.float32)
    xb = wl.f32_to_bf16_bits(x)
    assert np.array_equal(wl.bf16_bits_to_f32(xb), x)
    codes, bs, bz = _quant_block(oracle, xb)
    assert np.array_equal(codes, k.astype(np.uint8))
    out = np.full(x.shape, np.nan)
    tok = np.arange(32, dtype=np.int64).reshape(1, 32)
    oracle.dequantize_k_channel(codes, tok, bs, bz, out)
    assert np.array_equal(out, x.astype(np.float64))
    # random data: half-step bound per channel
    xb = _random_tokens(rng, 32, 2, "outlier")
    codes, bs, bz = _quant_block(oracle, xb)
    out = np.full(xb.shape, np.nan)
    oracle.dequantize_k_channel(codes, tok, bs, bz, out)
    x = wl.bf16_bits_to_f32(xb).astype(np.float64)
    s = bs.view(np.float16).astype(np.float64)
    bound = s / 2 * (1 + 2.0 ** -10) + 3 * 2.0 ** -11 * s
    assert np.all(np.abs(out - x) <= bound)
    # rows outside the listed blocks are left alone
    out = np.full((40, 2, 128), 7.0)
    c40 = np.zeros((40, 2, 128), np.uint8)
    c40[4:36] = codes
    oracle.dequantize_k_channel(c40, tok + 4, bs, bz, out)
    assert np.all(out[:4] == 7.0) and np.all(out[36:] == 7.0) and np.array_equal(out[4:36], codes * s + bz.view(np.float16).astype(np.float64))


def test_blocks_are_independent(oracle):
    rng = np.random.default_rng(405)
    xb = _random_tokens(rng, 64, 1, "normal")
    a = _quant_block(oracle, xb)
    y = xb.copy()
    y[40, 0, 9] = wl.f32_to_bf16_bits(np.float32([99.0]))[0]
    b = _quant_block(oracle, y)
    assert np.array_equal(a[0][:32], b[0][:32]) and np.array_equal(a[1][0], b[1][0]) and np.array_equal(a[2][0], b[2][0])
    ch = (a[0][32:] != b[0][32:]).any(axis=(0, 1))
    assert ch[9] and ch.sum() == 1
    assert (a[1][1] != b[1][1]).sum() == 1 and a[1][1, 0, 9] != b[1][1, 0, 9]


def test_metadata_positions(oracle):
    """Positions derived by hand from the layout rule: per block 128 fp16, chunks of 8 per (group c/32,
    quarter 2*((c%32)/16) + (c%8)/4), the pair (c, c+8) of k = c%4 at 2k and 2k+1."""
    want = {(0, 0): 0, (0, 8): 1, (0, 1): 2, (0, 9): 3, (0, 3): 6, (0, 11): 7, (0, 4): 8, (0, 12): 9,
            (0, 7): 14, (0, 15): 15, (0, 16): 16, (0, 24): 17, (0, 20): 24, (0, 31): 31, (0, 32): 32,
            (0, 127): 127, (1, 0): 128, (1, 45): 128 + 32 + 8 + 3, (1, 127): 255}
    for (blk, c), idx in want.items():
        assert oracle.kcmeta_index(blk, c) == idx, (blk, c)
    assert sorted(oracle.kcmeta_index(b, c) for b in range(2) for c in range(128)) == list(range(256))


def test_block_metadata_codec_round_trip_and_extent(oracle):
    rng = np.random.default_rng(406)
    Hkv, P2, P4 = 2, 3, 2
    pool = rng.integers(0, 256, oracle.pool_bytes(Hkv, P2, P4), dtype=np.uint8)
    before = pool.copy()
    bs = rng.integers(0, 65536, (2, Hkv, 128)).astype(np.uint16)
    bz = rng.integers(0, 65536, (2, Hkv, 128)).astype(np.uint16)
    slot_ids = np.concatenate([2 * 64 + np.arange(64)]).astype(np.int64)      # page 2, both blocks
    tok = np.arange(64, dtype=np.int64).reshape(2, 32)
    oracle.put_kblocks(pool, Hkv, P2, slot_ids, tok, bs, bz)
    gs, gz = oracle.get_kblocks(pool, Hkv, P2, slot_ids, tok)
    assert np.array_equal(gs, bs) and np.array_equal(gz, bz)
    changed = np.flatnonzero(pool != before)
    for h in range(Hkv):
        off, bits = oracle.record_offset(Hkv, P2, 2, h)
        assert bits == 2
    lo = oracle.record_offset(Hkv, P2, 2, 0)[0]
    # K scale and K zero planes follow the 2048 bytes of K codes in an INT2 record
    rel = (changed - lo) % oracle.record_bytes(2)
    assert changed.min() >= lo and np.all((rel >= 2048) & (rel < 2048 + 1024))
    # block 0 occupies the first half of each plane, block 1 the second
    pool2 = before.copy()
    oracle.put_kblocks(pool2, Hkv, P2, slot_ids, tok[:1], bs[:1], bz[:1])
    rel = (np.flatnonzero(pool2 != before) - lo) % oracle.record_bytes(2)
    assert np.all(((rel >= 2048) & (rel < 2048 + 256)) | ((rel >= 2560) & (rel < 2560 + 256)))


def test_residual_policy(oracle):
    """Sec. 3.2.1, residual policy: INT2-tagged tokens that do not fill a group of 32 go to INT4."""
    b = np.uint8([2] * 64)
    assert np.array_equal(oracle.route_residual(b), b)
    b = np.uint8([2] * 31)
    assert np.array_equal(oracle.route_residual(b), np.uint8([4] * 31))
    b = np.uint8([4, 2] * 37)                      # 37 INT2 tokens at odd positions
    r = oracle.route_residual(b)
    assert np.array_equal(r[0::2], b[0::2])        # INT4 tokens keep their width
    assert r[1::2].tolist() == [2] * 32 + [4] * 5  # the LAST five INT2 tokens are the residual
    rng = np.random.default_rng(407)
    for _ in range(50):
        b = rng.choice([2, 4], int(rng.integers(0, 300))).astype(np.uint8)
        r = oracle.route_residual(b)
        n2 = int((b == 2).sum())
        assert int((r == 2).sum()) == n2 // 32 * 32 and np.all(r[b == 4] == 4)
        assert np.all(np.diff((r == 4)[b == 2].astype(int)) >= 0)      # a suffix of the INT2 tokens
        blocks = oracle.int2_blocks(r, base=10)
        assert blocks.shape == (n2 // 32, 32) and np.array_equal(blocks.ravel() - 10, np.flatnonzero(r == 2))


def test_bad_arguments_are_rejected(oracle):
    x = np.zeros((32, 1, 128), np.uint16)
    codes = np.zeros((32, 1, 128), np.uint8)
    with pytest.raises(ValueError):
        oracle.quantize_k_channel(x, np.arange(32, dtype=np.int64).reshape(1, 32) + 1, codes)
    with pytest.raises(ValueError):
        oracle.quantize_k_channel(x, np.arange(32, dtype=np.int64).reshape(1, 32), codes, bits=3)
