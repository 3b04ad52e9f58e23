"""Shared helpers of the GPU parity tests: run a workload through the HIP
library (via the harness) and through the CPU oracle on the same seeded
inputs."""
import math

import numpy as np
import torch

from oracle import tkv_oracle as orc
from paper_2605_17170_amd import harness, tkv
from paper_2605_17170_amd import workloads as wl

DEV = "cuda:0"
SM = float(np.float32(1.0 / math.sqrt(128.0)))
ATOL, RTOL = 2e-3, 1e-2      # the parity tolerance of the decode output: |gpu - ref| <= ATOL + RTOL*|ref|


def oracle_pool(cache, Kq, Vq, fill):
    """Pack the oracle's canonical arrays into a host pool with the plan's slots."""
    pool = np.full(tkv.tkv_pool_bytes(cache.desc), fill, np.uint8)
    bmap = np.zeros(cache.P2 + cache.P4, np.uint8)
    orc.pack_pool(pool, bmap, cache.n_kv_heads, cache.P2, cache.P4, cache.slot_ids.astype(np.int64),
                  cache.tag_bits, Kq, Vq)
    return pool, bmap


def gpu_append(cache, K, V):
    dK, dV = harness.bf16_tensor(K, DEV), harness.bf16_tensor(V, DEV)
    cache.append(dK, dV)
    torch.cuda.synchronize()
    assert int(cache.status.item()) == 0
    return cache.pool.cpu().numpy(), cache.bit_map.cpu().numpy()


def check_append(seq_bits, K, V, n_kv_heads, fill=0xA5, pool_factor=1.5, shuffle_seed=3):
    """GPU append vs oracle quantise + pack: canonical arrays, then every pool byte."""
    cache = harness.PagedCache(n_kv_heads, seq_bits, DEV, pool_factor=pool_factor, shuffle_seed=shuffle_seed, fill=fill)
    try:
        g_pool, g_map = gpu_append(cache, K, V)
        bits = cache.tag_bits
        Kq, Vq = orc.quantize(K, bits), orc.quantize(V, bits)
        gK, gV = orc.unpack_pool(g_pool, n_kv_heads, cache.P2, cache.P4, cache.slot_ids.astype(np.int64))
        names = ["K codes", "K scale", "K zero", "V codes", "V scale", "V zero"]
        for name, a, b in zip(names, gK + gV, Kq + Vq):
            bad = np.argwhere(a != b)
            assert bad.size == 0, "%s differ at %s: gpu %s oracle %s" % (name, bad[:4].tolist(), a[tuple(bad[0])], b[tuple(bad[0])])
        o_pool, o_map = oracle_pool(cache, Kq, Vq, fill)
        assert np.array_equal(g_map, o_map)
        diff = np.nonzero(g_pool != o_pool)[0]
        assert diff.size == 0, "pool bytes differ at %s" % diff[:8].tolist()
        return cache, (Kq, Vq)
    except Exception:
        cache.close()
        raise


def assert_close(got, ref, what=""):
    got = np.asarray(got, np.float64)
    err = np.abs(got - ref)
    tol = ATOL + RTOL * np.abs(ref)
    assert np.all(np.isfinite(got)), what + ": non-finite output"
    worst = np.unravel_index(np.argmax(err - tol), err.shape)
    assert np.all(err <= tol), "%s: |gpu-ref|=%.3e > tol %.3e at %s (ref %.5f)" % (what, err[worst], tol[worst], worst, ref[worst])
    ratio = float((err / tol).max())
    print("  parity %s: max |gpu-ref|/tol = %.4f, max abs err %.3e" % (what, ratio, float(err.max())), flush=True)
    return ratio


def decode_ref(q, Kq, Vq, seq_lens):
    ip = np.concatenate([[0], np.cumsum(seq_lens)]).astype(np.int64)
    return orc.attention_quantized(q, Kq, Vq, ip, SM)


def gpu_decode(cache, q, target_items, expect_status=0):
    cache.plan_decode(target_items)
    dq = harness.bf16_tensor(q, DEV)
    out = cache.decode(dq)
    torch.cuda.synchronize()
    assert int(cache.status.item()) == expect_status
    return out.cpu().numpy()


def random_case(seed, seq_lens, n_q_heads, n_kv_heads, f4=0.4, run=37):
    """Random K/V/q with outlier channels and a per-token width pattern made of
    runs (so that both page streams get partial pages)."""
    ss = np.random.SeedSequence([seed, 99])
    s_kv, s_q, s_b = ss.spawn(3)
    rng = np.random.default_rng(s_b)
    T = int(np.sum(seq_lens))
    K, V, _ = wl.make_kv(s_kv, T, n_kv_heads)
    q = wl.make_q(s_q, len(seq_lens), n_q_heads)
    seq_bits = []
    for n in seq_lens:
        b = np.empty(n, np.uint8)
        pos = 0
        while pos < n:
            ln = int(rng.integers(1, run + 1))
            b[pos:pos + ln] = 4 if rng.random() < f4 else 2
            pos += ln
        seq_bits.append(b)
    return q, K, V, seq_bits


# ------------------------------------------------------------------ per-channel INT2 keys (Sec. 3.2.1)
def kc_oracle(seq_bits, K, V):
    """Oracle side of a cache with per-channel INT2 keys, from the ORIGINAL per-token tags: residual policy,
    per-token quantisation (V everywhere, K of the INT4 tokens), per-channel quantisation of the INT2 key
    blocks.  Returns (bits, Kq, Vq, tok_blocks, bscale, bzero)."""
    routed = [orc.route_residual(b) for b in seq_bits]
    bits = np.concatenate(routed) if routed else np.zeros(0, np.uint8)
    Kq, Vq = orc.quantize(K, bits), orc.quantize(V, bits)
    base, blocks = 0, []
    for b in routed:
        blocks.append(orc.int2_blocks(b, base))
        base += b.size
    tok = np.concatenate(blocks) if blocks else np.zeros((0, 32), np.int64)
    bs, bz = orc.quantize_k_channel(K, tok, Kq[0])      # overwrites the codes of the INT2 rows
    i2 = bits == 2
    Kq[1][i2] = 0                                        # no per-token key metadata for those rows
    Kq[2][i2] = 0
    return bits, Kq, Vq, tok, bs, bz


def kc_oracle_pool(cache, Kq, Vq, tok, bs, bz, fill):
    pool, bmap = oracle_pool(cache, Kq, Vq, fill)
    orc.put_kblocks(pool, cache.n_kv_heads, cache.P2, cache.slot_ids.astype(np.int64), tok, bs, bz)
    return pool, bmap


def kc_dequantized(Kq, Vq, tok, bs, bz):
    Kh = orc.dequantize(*Kq)
    orc.dequantize_k_channel(Kq[0], tok, bs, bz, Kh)
    return Kh, orc.dequantize(*Vq)


def kc_check_append(seq_bits, K, V, n_kv_heads, fill=0xA5, pool_factor=1.5, shuffle_seed=3):
    """GPU append with per-channel INT2 keys vs the oracle: routing, codes, block metadata, every pool byte."""
    cache = harness.PagedCache(n_kv_heads, seq_bits, DEV, pool_factor=pool_factor, shuffle_seed=shuffle_seed, fill=fill,
                               key_axis=tkv.TKV_KEYS_PER_CHANNEL)
    try:
        bits, Kq, Vq, tok, bs, bz = kc_oracle(seq_bits, K, V)
        assert np.array_equal(cache.tag_bits, bits), "residual routing differs"
        g_pool, g_map = gpu_append(cache, K, V)
        slots = cache.slot_ids.astype(np.int64)
        gK, gV = orc.unpack_pool(g_pool, n_kv_heads, cache.P2, cache.P4, slots)
        i4 = bits == 4
        assert np.array_equal(gK[0], Kq[0]), "K codes differ at %s" % np.argwhere(gK[0] != Kq[0])[:4].tolist()
        assert np.array_equal(gK[1][i4], Kq[1][i4]) and np.array_equal(gK[2][i4], Kq[2][i4])
        gs, gz = orc.get_kblocks(g_pool, n_kv_heads, cache.P2, slots, tok)
        assert np.array_equal(gs, bs), "block scales differ at %s" % np.argwhere(gs != bs)[:4].tolist()
        assert np.array_equal(gz, bz), "block zeros differ at %s" % np.argwhere(gz != bz)[:4].tolist()
        for name, a, b in zip(["V codes", "V scale", "V zero"], gV, Vq):
            assert np.array_equal(a, b), name
        o_pool, o_map = kc_oracle_pool(cache, Kq, Vq, tok, bs, bz, fill)
        assert np.array_equal(g_map, o_map)
        diff = np.nonzero(g_pool != o_pool)[0]
        assert diff.size == 0, "pool bytes differ at %s" % diff[:8].tolist()
        return cache, (bits, Kq, Vq, tok, bs, bz)
    except Exception:
        cache.close()
        raise


def kc_decode_ref(q, ref, seq_lens):
    bits, Kq, Vq, tok, bs, bz = ref
    Kh, Vh = kc_dequantized(Kq, Vq, tok, bs, bz)
    ip = np.concatenate([[0], np.cumsum(seq_lens)]).astype(np.int64)
    return orc.attention_f64(wl.bf16_bits_to_f32(q).astype(np.float64), Kh, Vh, ip, SM)
