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


def gpu_decode(cache, q, target_items):
    cache.plan_decode(target_items)
    dq = harness.bf16_tensor(q, DEV)
    out = cache.decode(dq)
    torch.cuda.synchronize()
    assert int(cache.status.item()) == 0
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
