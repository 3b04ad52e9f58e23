"""Pins for the oracle's page codec: hand-derived positions, bijectivity of
every plane, the structural rules of the layout, pack/unpack identity and
non-interference with bits that belong to other slots."""
import os

import numpy as np
import pytest

from paper_2605_17170_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden", "layout_positions.txt")


def test_hand_derived_positions(oracle):
    n = 0
    for line in open(GOLD):
        line = line.split("#")[0].split()
        if not line:
            continue
        plane, bits, t, c, word, shift = line[0], *map(int, line[1:])
        if plane == "K":
            assert oracle.kcode_pos(bits, t, c) == (word, shift), line
        elif plane == "V":
            assert oracle.vcode_pos(bits, t, c) == (word, shift), line
        elif plane == "KM":
            assert oracle.kmeta_index(t, c) == word, line
        else:
            assert oracle.vmeta_index(t, c) == word, line
        n += 1
    assert n >= 50


@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("plane", ["K", "V"])
def test_code_planes_are_bijective(oracle, bits, plane):
    pos = oracle.kcode_pos if plane == "K" else oracle.vcode_pos
    seen = set()
    for t in range(64):
        for c in range(128):
            w, s = pos(bits, t, c)
            assert 0 <= w < 64 * 128 * bits // 32 and s % bits == 0 and 0 <= s <= 32 - bits
            seen.add((w, s))
    assert len(seen) == 64 * 128


def test_meta_planes_are_bijective(oracle):
    assert sorted(oracle.kmeta_index(t, g) for t in range(64) for g in range(4)) == list(range(256))
    assert sorted(oracle.vmeta_index(t, g) for t in range(64) for g in range(4)) == list(range(256))


@pytest.mark.parametrize("bits", [2, 4])
def test_layout_structure(oracle, bits):
    per_word = 32 // bits
    # K: a word holds consecutive channels of ONE group of ONE token; the four
    # words of a 16-byte chunk are the four groups of the same channel slice.
    for t in (0, 5, 63):
        for c0 in range(0, 128, per_word):
            ws = {oracle.kcode_pos(bits, t, c0 + k) for k in range(per_word)}
            assert len({w for w, _ in ws}) == 1
            assert sorted(s for _, s in ws) == list(range(0, 32, bits))
        for cg in range(32):
            words = [oracle.kcode_pos(bits, t, 32 * g + cg)[0] for g in range(4)]
            assert words[0] % 4 == 0 and words == [words[0] + g for g in range(4)]
    # a 16-token tile of K codes is one contiguous block of the plane
    tile_words = 16 * 128 * bits // 32
    for tile in range(4):
        ws = {oracle.kcode_pos(bits, 16 * tile + r, c)[0] for r in range(16) for c in range(128)}
        assert ws == set(range(tile * tile_words, (tile + 1) * tile_words))
    # V: a word holds ONE channel and tokens that share (t % 16) // 4
    for c in (0, 17, 127):
        by_word = {}
        for t in range(64):
            w, s = oracle.vcode_pos(bits, t, c)
            by_word.setdefault(w, []).append(t)
        assert all(len(v) == per_word for v in by_word.values())
        for toks in by_word.values():
            assert len({(t % 16) // 4 for t in toks}) == 1
            if bits == 4:
                assert len({t // 32 for t in toks}) == 1
    # V metadata lists tokens in the order in which a V word lists them:
    # tokens 2k and 2k+1 of a metadata chunk sit in the low / high half of
    # the same 16-bit-pair position of the code word
    for t in range(64):
        j = oracle.vmeta_index(t, 0) % 8
        shift = oracle.vcode_pos(bits, t, 0)[1]
        assert (shift >= 16) == (j % 2 == 1)


def test_sizes(oracle):
    assert oracle.record_bytes(2) == 6144 and oracle.record_bytes(4) == 10240
    # 96 / 160 bytes per token and kv head: 3.0 / 5.0 bits per element, so an
    # average of 2.6 code bits costs 3.6 bits and gives 16/3.6 = 4.4x over
    # bf16, the capacity figure of the paper's abstract
    assert oracle.record_bytes(2) // 64 == 96 and oracle.record_bytes(4) // 64 == 160
    assert oracle.pool_bytes(8, 10, 20) == 8 * (10 * 6144 + 20 * 10240)
    assert oracle.record_offset(8, 10, 3, 5) == ((3 * 8 + 5) * 6144, 2)
    assert oracle.record_offset(8, 10, 12, 1) == (10 * 8 * 6144 + (2 * 8 + 1) * 10240, 4)


def _canon(rng, T, H, bits):
    hi = np.where(bits == 2, 4, 16)[:, None, None]
    Kc = (rng.integers(0, 16, (T, H, 128)) % hi).astype(np.uint8)
    Vc = (rng.integers(0, 16, (T, H, 128)) % hi).astype(np.uint8)
    meta = [rng.integers(0, 65536, (T, H, 4)).astype(np.uint16) for _ in range(4)]
    return (Kc, meta[0], meta[1]), (Vc, meta[2], meta[3])


def test_pack_unpack_identity_and_canary(oracle):
    rng = np.random.default_rng(3)
    H, P2, P4 = 3, 5, 4
    T = 300
    bits = rng.choice([2, 4], T).astype(np.uint8)
    # random distinct slots inside the matching pool
    s2 = rng.permutation(P2 * 64)[: int((bits == 2).sum())]
    s4 = rng.permutation(P4 * 64)[: int((bits == 4).sum())] + P2 * 64
    assert s2.size == (bits == 2).sum() and s4.size == (bits == 4).sum()
    slots = np.empty(T, np.int64)
    slots[bits == 2] = s2
    slots[bits == 4] = s4
    Kq, Vq = _canon(rng, T, H, bits)
    nbytes = oracle.pool_bytes(H, P2, P4)
    pool = np.full(nbytes, 0xA5, np.uint8)
    bmap = np.zeros(P2 + P4, np.uint8)
    oracle.pack_pool(pool, bmap, H, P2, P4, slots, bits, Kq, Vq)
    Kq2, Vq2 = oracle.unpack_pool(pool, H, P2, P4, slots)
    for a, b in zip(Kq + Vq, Kq2 + Vq2):
        assert np.array_equal(a, b)
    touched = np.unique(slots // 64)
    assert np.array_equal(np.nonzero(bmap)[0], touched)
    assert np.all(bmap[touched] == np.where(touched < P2, 2, 4))
    # slots never written still read back as the 0xA5 canary pattern
    free = np.setdiff1d(np.arange((P2 + P4) * 64), slots)
    Kf, Vf = oracle.unpack_pool(pool, H, P2, P4, free)
    fb = np.where(free < P2 * 64, 2, 4)
    want_code = np.where(fb == 2, 0xA5 & 3, 0xA5 & 15)  # 0b10100101: crumbs 1, nibble 5
    assert np.all(Kf[1] == 0xA5A5) and np.all(Vf[2] == 0xA5A5)
    # INT2 crumbs of 0xA5 are 1,1,2,2 depending on position, INT4 nibbles 5 or 10
    assert set(np.unique(Kf[0][fb == 2])) <= {1, 2} and set(np.unique(Kf[0][fb == 4])) <= {5, 10}
    assert want_code.size == free.size
    # overwriting with other data changes only the written slots
    pool2 = pool.copy()
    Kq3, Vq3 = _canon(rng, T, H, bits)
    oracle.pack_pool(pool2, bmap, H, P2, P4, slots, bits, Kq3, Vq3)
    Kf2, Vf2 = oracle.unpack_pool(pool2, H, P2, P4, free)
    for a, b in zip(Kf + Vf, Kf2 + Vf2):
        assert np.array_equal(a, b)


def test_pack_rejects_width_mismatch(oracle):
    H, P2, P4 = 1, 1, 1
    pool = np.zeros(oracle.pool_bytes(H, P2, P4), np.uint8)
    bmap = np.zeros(2, np.uint8)
    Kq, Vq = _canon(np.random.default_rng(0), 1, H, np.uint8([2]))
    with pytest.raises(ValueError):
        oracle.pack_pool(pool, bmap, H, P2, P4, np.int64([64]), np.uint8([2]), Kq, Vq)  # slot 64 is in the INT4 pool
