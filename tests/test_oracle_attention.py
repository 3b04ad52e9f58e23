"""Pins for the oracle's attention (paper Sec. 3.2.3 "Decode": the split
flash-decoding result equals softmax(q K^T / sqrt(d)) V over the dequantised
cache).  Checked against torch's fp64 scaled_dot_product_attention, a
pure-Python brute force, closed forms and invariances."""
import math

import numpy as np
import pytest
import torch

from paper_2605_17170_amd import workloads as wl

SM = 1.0 / math.sqrt(128.0)


def _torch_ref(q, K, V, indptr, sm_scale):
    B, Hq, D = q.shape
    Hkv = K.shape[1]
    R = Hq // Hkv
    out = np.zeros((B, Hq, D))
    for b in range(B):
        k = torch.from_numpy(K[indptr[b]:indptr[b + 1]]).permute(1, 0, 2)  # [Hkv, n, D]
        v = torch.from_numpy(V[indptr[b]:indptr[b + 1]]).permute(1, 0, 2)
        if k.shape[1] == 0:
            continue
        k = k.repeat_interleave(R, dim=0)
        v = v.repeat_interleave(R, dim=0)
        qq = torch.from_numpy(q[b])[:, None, :]
        o = torch.nn.functional.scaled_dot_product_attention(qq, k, v, scale=sm_scale)
        out[b] = o[:, 0, :].numpy()
    return out


def test_dense_attention_matches_torch_sdpa(oracle):
    rng = np.random.default_rng(1)
    B, Hq, Hkv, D = 3, 8, 2, 128
    lens = np.array([5, 130, 77])
    ip = np.concatenate([[0], np.cumsum(lens)])
    q = rng.standard_normal((B, Hq, D))
    K = rng.standard_normal((ip[-1], Hkv, D)) * 2
    V = rng.standard_normal((ip[-1], Hkv, D))
    got = oracle.attention_f64(q, K, V, ip, SM)
    want = _torch_ref(q, K, V, ip, SM)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-13)


def _exact_kv(rng, T, H, bits):
    """Values z + c*s with a power-of-two step and codes 0 and L present in
    every group: the quantiser must reproduce them bit for bit."""
    L = 2 ** bits - 1
    z, s = (-2.0, 0.25) if bits == 4 else (-1.0, 0.5)
    c = rng.integers(0, L + 1, (T, H, 4, 32))
    c[..., 0] = 0
    c[..., 1] = L
    c = rng.permuted(c, axis=-1)
    return (z + s * c).reshape(T, H, 128)


def test_exactly_representable_input_reproduces_unquantised_attention(oracle):
    rng = np.random.default_rng(2)
    B, Hq, Hkv = 2, 8, 2
    lens = np.array([200, 95])
    ip = np.concatenate([[0], np.cumsum(lens)])
    bits = rng.choice([2, 4], ip[-1]).astype(np.uint8)
    K = np.empty((ip[-1], Hkv, 128))
    V = np.empty((ip[-1], Hkv, 128))
    for b in (2, 4):
        K[bits == b] = _exact_kv(rng, int((bits == b).sum()), Hkv, b)
        V[bits == b] = _exact_kv(rng, int((bits == b).sum()), Hkv, b)
    Kb, Vb = wl.f32_to_bf16_bits(K.astype(np.float32)), wl.f32_to_bf16_bits(V.astype(np.float32))
    assert np.array_equal(wl.bf16_bits_to_f32(Kb).astype(np.float64), K)
    qb = wl.normal_bf16(rng, (B, Hq, 128))
    Kq, Vq = oracle.quantize(Kb, bits), oracle.quantize(Vb, bits)
    assert np.array_equal(oracle.dequantize(*Kq), K) and np.array_equal(oracle.dequantize(*Vq), V)
    got = oracle.attention_quantized(qb, Kq, Vq, ip, SM)
    qf = wl.bf16_bits_to_f32(qb).astype(np.float64)
    want = _torch_ref(qf, K, V, ip, SM)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-13)


def test_quantised_attention_is_dense_attention_on_dequantised_cache(oracle):
    rng = np.random.default_rng(3)
    B, Hq, Hkv = 2, 4, 1
    lens = np.array([300, 64])
    ip = np.concatenate([[0], np.cumsum(lens)])
    bits = rng.choice([2, 4], ip[-1]).astype(np.uint8)
    K, V, _ = wl.make_kv(np.random.SeedSequence(9), int(ip[-1]), Hkv)
    qb = wl.make_q(np.random.SeedSequence(10), B, Hq)
    Kq, Vq = oracle.quantize(K, bits), oracle.quantize(V, bits)
    got = oracle.attention_quantized(qb, Kq, Vq, ip, SM)
    want = _torch_ref(wl.bf16_bits_to_f32(qb).astype(np.float64), oracle.dequantize(*Kq), oracle.dequantize(*Vq), ip, SM)
    assert np.allclose(got, want, rtol=1e-11, atol=1e-12)


def test_brute_force_tiny_heads(oracle):
    """Pure-Python loops on a handful of tokens, including the grouped-query
    head mapping h -> h // (Hq/Hkv)."""
    rng = np.random.default_rng(4)
    B, Hq, Hkv, D = 2, 4, 2, 128
    lens = [3, 2]
    ip = np.array([0, 3, 5])
    q = rng.standard_normal((B, Hq, D))
    K = rng.standard_normal((5, Hkv, D))
    V = rng.standard_normal((5, Hkv, D))
    got = oracle.attention_f64(q, K, V, ip, 0.3)
    for b in range(B):
        for h in range(Hq):
            kh = h // 2
            logits = []
            for t in range(ip[b], ip[b + 1]):
                logits.append(0.3 * math.fsum(float(q[b, h, c]) * float(K[t, kh, c]) for c in range(D)))
            w = [math.exp(l - max(logits)) for l in logits]
            for c in range(D):
                o = math.fsum(wi * float(V[ip[b] + i, kh, c]) for i, wi in enumerate(w)) / math.fsum(w)
                assert abs(got[b, h, c] - o) < 1e-12
    assert lens == [3, 2]


def test_closed_forms(oracle):
    rng = np.random.default_rng(5)
    D = 128
    q = rng.standard_normal((1, 1, D))
    # one token: out = V
    K = rng.standard_normal((1, 1, D))
    V = rng.standard_normal((1, 1, D))
    assert np.allclose(oracle.attention_f64(q, K, V, [0, 1], SM)[0, 0], V[0, 0], rtol=0, atol=1e-15)
    # identical keys: uniform weights -> mean of V
    K = np.repeat(K, 7, axis=0)
    V = rng.standard_normal((7, 1, D))
    assert np.allclose(oracle.attention_f64(q, K, V, [0, 7], SM)[0, 0], V[:, 0].mean(0), atol=1e-14)
    # two tokens with logit gap d: weights sigmoid(+-d)
    K = rng.standard_normal((2, 1, D))
    V = rng.standard_normal((2, 1, D))
    d = SM * float(q[0, 0] @ (K[0, 0] - K[1, 0]))
    w0 = 1.0 / (1.0 + math.exp(-d))
    want = w0 * V[0, 0] + (1 - w0) * V[1, 0]
    assert np.allclose(oracle.attention_f64(q, K, V, [0, 2], SM)[0, 0], want, atol=1e-14)


def test_empty_sequence_gives_zeros_and_order_does_not_matter(oracle):
    rng = np.random.default_rng(6)
    q = rng.standard_normal((2, 2, 128))
    K = rng.standard_normal((50, 1, 128))
    V = rng.standard_normal((50, 1, 128))
    out = oracle.attention_f64(q, K, V, [0, 0, 50], SM)
    assert np.all(out[0] == 0) and np.all(np.isfinite(out))
    perm = rng.permutation(50)
    out2 = oracle.attention_f64(q, K[perm], V[perm], [0, 0, 50], SM)
    assert np.allclose(out, out2, rtol=1e-12, atol=1e-14)


def test_large_logits_do_not_overflow(oracle):
    q = np.full((1, 1, 128), 30.0)
    K = np.stack([np.full((1, 128), 30.0), np.full((1, 128), -30.0)])
    V = np.stack([np.full((1, 128), 1.0), np.full((1, 128), 5.0)])
    out = oracle.attention_f64(q, K, V, [0, 2], 1.0)
    assert np.allclose(out, 1.0)


def test_fp32_reevaluation_is_far_inside_the_parity_tolerance(oracle):
    """The 2e-3 + 1e-2*|ref| parity tolerance is about the GPU's fp32
    summation order, not about the reference: an fp32 evaluation of the same
    definition sits orders of magnitude inside it."""
    w = wl.config("cfg1")
    q, K, V, _ = w.make_inputs()
    bits = w.all_bits()
    Kq, Vq = oracle.quantize(K, bits), oracle.quantize(V, bits)
    ref = oracle.attention_quantized(q, Kq, Vq, w.seq_indptr, SM)
    Kh = torch.from_numpy(oracle.dequantize(*Kq)).float()
    Vh = torch.from_numpy(oracle.dequantize(*Vq)).float()
    qf = torch.from_numpy(wl.bf16_bits_to_f32(q))
    logits = torch.einsum("hd,td->ht", qf[0], Kh[:, 0]) * np.float32(SM)
    o32 = (torch.softmax(logits, -1) @ Vh[:, 0]).numpy()
    err = np.abs(o32 - ref[0])
    assert np.all(err <= 0.05 * (2e-3 + 1e-2 * np.abs(ref[0])))
