"""ctypes front end of the CPU oracle (oracle/tkv_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
CPU-baseline leg of the benchmark.  The product package never imports this
module and this module never imports the product package.

Every function takes and returns numpy arrays; bf16 / fp16 values travel as
uint16 bit patterns.  Shapes follow the paper's notation: T tokens, Hkv
key/value heads, Hq query heads, D = head_dim, G = group size (Sec. 3.2.1).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tkv_oracle.c")
_LIB = os.path.join(_HERE, "libtkv_oracle.so")

TP, HD, GS, NG = 64, 128, 32, 4


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fused multiply-add, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-shared", "-fPIC", "-Wall", "-Wextra", "-o", _LIB + ".tmp", _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(_LIB + ".tmp", _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        L = _lib
        L.tkvo_record_bytes.restype = C.c_int64
        L.tkvo_pool_bytes.restype = C.c_int64
        L.tkvo_pool_bytes.argtypes = [C.c_int, C.c_int64, C.c_int64]
        L.tkvo_record_offset.restype = C.c_int64
        L.tkvo_record_offset.argtypes = [C.c_int, C.c_int64, C.c_int64, C.c_int, C.c_void_p]
        L.tkvo_bf16_to_f32.restype = C.c_float
        L.tkvo_f16_to_f32.restype = C.c_float
        L.tkvo_f32_to_f16.restype = C.c_uint16
        L.tkvo_f32_to_f16.argtypes = [C.c_float]
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def num_threads() -> int:
    return int(lib().tkvo_num_threads())


# ---------------------------------------------------------------- formats
def bf16_to_f32(x_u16):
    x = _c(x_u16, np.uint16)
    out = np.empty(x.shape, np.float32)
    lib().tkvo_bf16_to_f32_array(_p(x), _p(out), C.c_int64(x.size))
    return out


def f16_to_f32(x_u16):
    x = _c(x_u16, np.uint16)
    out = np.empty(x.shape, np.float32)
    lib().tkvo_f16_to_f32_array(_p(x), _p(out), C.c_int64(x.size))
    return out


def f32_to_f16(x_f32):
    x = _c(x_f32, np.float32)
    out = np.empty(x.shape, np.uint16)
    lib().tkvo_f32_to_f16_array(_p(x), _p(out), C.c_int64(x.size))
    return out


# ---------------------------------------------------------------- quantiser
def f64_to_f16(x_f64):
    """binary64 -> binary16 bit patterns, nearest-even, one rounding."""
    x = _c(x_f64, np.float64)
    out = np.empty(x.shape, np.uint16)
    lib().tkvo_f64_to_f16_array(_p(x), _p(out), C.c_int64(x.size))
    return out


def quantize_group(x_u16, bits: int):
    """One group of G channels -> (codes u8[G], scale u16, zero u16)."""
    x = _c(x_u16, np.uint16)
    codes = np.empty(x.size, np.uint8)
    s = C.c_uint16(0)
    z = C.c_uint16(0)
    lib().tkvo_quantize_group(_p(x), C.c_int(x.size), C.c_int(bits), _p(codes), C.byref(s), C.byref(z))
    return codes, int(s.value), int(z.value)


def quantize(x_u16, bits_u8, G: int = GS):
    """x: bf16 bits [T, H, D]; bits: u8 [T].  Returns codes u8 [T,H,D],
    scale u16 [T,H,D/G], zero u16 [T,H,D/G] (Sec. 3.2.1, per-token groups)."""
    x = _c(x_u16, np.uint16)
    bits = _c(bits_u8, np.uint8)
    T, H, D = x.shape
    assert bits.shape == (T,)
    codes = np.empty((T, H, D), np.uint8)
    scale = np.empty((T, H, D // G), np.uint16)
    zero = np.empty((T, H, D // G), np.uint16)
    rc = lib().tkvo_quantize(_p(x), C.c_int64(T), C.c_int(H), C.c_int(D), C.c_int(G), _p(bits),
                             _p(codes), _p(scale), _p(zero))
    if rc:
        raise ValueError("oracle quantize: bad bitwidth or shape")
    return codes, scale, zero


def dequantize(codes, scale, zero, G: int = GS):
    codes = _c(codes, np.uint8)
    scale = _c(scale, np.uint16)
    zero = _c(zero, np.uint16)
    T, H, D = codes.shape
    out = np.empty((T, H, D), np.float64)
    lib().tkvo_dequantize(_p(codes), _p(scale), _p(zero), C.c_int64(T), C.c_int(H), C.c_int(D), C.c_int(G), _p(out))
    return out


# ------------------------------------------------- per-channel INT2 keys (Sec. 3.2.1)
def route_residual(bits_u8, G: int = GS):
    """Residual policy for INT2 keys (Sec. 3.2.1): per-channel quantisation needs whole groups of G tokens,
    so the INT2-tagged tokens of one arriving sequence chunk that do not fill a group -- the last
    (count mod G) of them -- take the INT4 per-token path.  Returns the rewritten per-token bitwidth array."""
    bits = np.array(bits_u8, np.uint8, copy=True)
    idx = np.flatnonzero(bits == 2)
    r = idx.size % G
    if r:
        bits[idx[idx.size - r:]] = 4
    return bits


def int2_blocks(bits_u8, base: int = 0, G: int = GS):
    """Token rows of the groups of G INT2 tokens, in arrival order: i64 [nb, G] (rows offset by `base`)."""
    idx = np.flatnonzero(np.asarray(bits_u8) == 2)
    assert idx.size % G == 0, "route_residual first"
    return (idx.reshape(-1, G) + base).astype(np.int64)


def quantize_k_channel(x_u16, tok_blocks, codes_out, bits: int = 2):
    """Keys quantised per channel over blocks of G tokens.  x: bf16 bits [T,H,D]; tok_blocks i64 [nb,G];
    codes_out u8 [T,H,D] receives the codes of the listed rows.  Returns (bscale, bzero) u16 [nb,H,D]."""
    x = _c(x_u16, np.uint16)
    tok = _c(tok_blocks, np.int64)
    T, H, D = x.shape
    nb, G = tok.shape if tok.ndim == 2 else (0, GS)
    assert codes_out.dtype == np.uint8 and codes_out.flags.c_contiguous and codes_out.shape == x.shape
    bs = np.empty((nb, H, D), np.uint16)
    bz = np.empty((nb, H, D), np.uint16)
    rc = lib().tkvo_quantize_k_channel(_p(x), C.c_int64(T), C.c_int(H), C.c_int(D), C.c_int(G), C.c_int(bits),
                                       _p(tok), C.c_int64(nb), _p(codes_out), _p(bs), _p(bz))
    if rc:
        raise ValueError("oracle quantize_k_channel: bad argument")
    return bs, bz


def dequantize_k_channel(codes, tok_blocks, bscale, bzero, out_f64):
    """x_hat = code * scale + zero (exact in fp64) written into the listed rows of out_f64 [T,H,D]."""
    tok = np.asarray(tok_blocks, np.int64)
    if tok.size == 0:
        return out_f64
    s = f16_to_f32(bscale).astype(np.float64)[:, None]     # [nb,1,H,D]
    z = f16_to_f32(bzero).astype(np.float64)[:, None]
    out_f64[tok] = codes[tok].astype(np.float64) * s + z   # rows [nb,G,H,D]
    return out_f64


def kcmeta_index(blk, c):
    return int(lib().tkvo_kcmeta_index(C.c_int(blk), C.c_int(c)))


def put_kblocks(pool_u8, Hkv, P2, slot_ids, tok_blocks, bscale, bzero):
    """Write the per-channel key metadata of every block into the record of the page its tokens sit in."""
    assert pool_u8.dtype == np.uint8 and pool_u8.flags.c_contiguous
    tok = np.asarray(tok_blocks, np.int64)
    bs, bz = _c(bscale, np.uint16), _c(bzero, np.uint16)
    for b in range(tok.shape[0]):
        sl = np.asarray(slot_ids)[tok[b]]
        page, slot0 = int(sl[0]) // TP, int(sl[0]) % TP
        assert slot0 % GS == 0 and np.array_equal(sl, sl[0] + np.arange(GS)) and page < P2
        for h in range(Hkv):
            off, _ = record_offset(Hkv, P2, page, h)
            rec = pool_u8[off:off + record_bytes(2)]
            lib().tkvo_record_put_kblock(_p(rec), C.c_int(slot0 // GS), _p(np.ascontiguousarray(bs[b, h])),
                                         _p(np.ascontiguousarray(bz[b, h])))


def get_kblocks(pool_u8, Hkv, P2, slot_ids, tok_blocks):
    """Read back (bscale, bzero) u16 [nb,H,D] of the listed blocks from a pool."""
    pool = _c(pool_u8, np.uint8)
    tok = np.asarray(tok_blocks, np.int64)
    nb = tok.shape[0]
    bs = np.empty((nb, Hkv, HD), np.uint16)
    bz = np.empty((nb, Hkv, HD), np.uint16)
    for b in range(nb):
        s0 = int(np.asarray(slot_ids)[tok[b, 0]])
        page, blk = s0 // TP, (s0 % TP) // GS
        for h in range(Hkv):
            off, _ = record_offset(Hkv, P2, page, h)
            rec = pool[off:off + record_bytes(2)]
            ks = np.empty(HD, np.uint16)
            kz = np.empty(HD, np.uint16)
            lib().tkvo_record_get_kblock(_p(rec), C.c_int(blk), _p(ks), _p(kz))
            bs[b, h], bz[b, h] = ks, kz
    return bs, bz


# ---------------------------------------------------------------- attention
def dequantize_f16(codes, scale, zero, G: int = GS):
    """The cached rows as FP16 bit patterns [T,H,D] (Sec. 3.2.3 "Prefill"): nearest-even of the exact
    code * scale + zero."""
    codes = _c(codes, np.uint8)
    scale = _c(scale, np.uint16)
    zero = _c(zero, np.uint16)
    T, H, D = codes.shape
    out = np.empty((T, H, D), np.uint16)
    lib().tkvo_dequantize_f16(_p(codes), _p(scale), _p(zero), C.c_int64(T), C.c_int(H), C.c_int(D), C.c_int(G), _p(out))
    return out


def attention_f64(q, K, V, seq_indptr, sm_scale: float):
    """Plain fp64 softmax(q K^T * sm_scale) V with grouped-query heads.
    q [B,Hq,D] f64; K,V [T,Hkv,D] f64; seq_indptr i64 [B+1]."""
    q = _c(q, np.float64)
    K = _c(K, np.float64)
    V = _c(V, np.float64)
    ip = _c(seq_indptr, np.int64)
    B, Hq, D = q.shape
    Hkv = K.shape[1]
    out = np.empty((B, Hq, D), np.float64)
    rc = lib().tkvo_attention_f64(_p(q), _p(K), _p(V), _p(ip), C.c_int(B), C.c_int(Hq), C.c_int(Hkv),
                                  C.c_int(D), C.c_double(sm_scale), _p(out))
    if rc:
        raise ValueError("oracle attention_f64 failed rc=%d" % rc)
    return out


def attention_quantized(q_u16, Kq, Vq, seq_indptr, sm_scale: float, G: int = GS):
    """Decode attention over the quantised cache (Sec. 3.2.3 "Decode").
    q: bf16 bits [B,Hq,D]; Kq, Vq: (codes, scale, zero) triples as returned by
    quantize(); tokens of all sequences concatenated in original order."""
    q = _c(q_u16, np.uint16)
    Kc, Ks, Kz = (_c(Kq[0], np.uint8), _c(Kq[1], np.uint16), _c(Kq[2], np.uint16))
    Vc, Vs, Vz = (_c(Vq[0], np.uint8), _c(Vq[1], np.uint16), _c(Vq[2], np.uint16))
    ip = _c(seq_indptr, np.int64)
    B, Hq, D = q.shape
    Hkv = Kc.shape[1]
    assert ip[-1] == Kc.shape[0]
    out = np.empty((B, Hq, D), np.float64)
    rc = lib().tkvo_attention_quantized(_p(q), _p(Kc), _p(Ks), _p(Kz), _p(Vc), _p(Vs), _p(Vz), _p(ip),
                                        C.c_int(B), C.c_int(Hq), C.c_int(Hkv), C.c_int(D), C.c_int(G),
                                        C.c_double(sm_scale), _p(out))
    if rc:
        raise ValueError("oracle attention_quantized failed rc=%d" % rc)
    return out


# ---------------------------------------------------------------- page codec
def record_bytes(bits: int) -> int:
    return int(lib().tkvo_record_bytes(C.c_int(bits)))


def pool_bytes(Hkv: int, P2: int, P4: int) -> int:
    return int(lib().tkvo_pool_bytes(Hkv, P2, P4))


def record_offset(Hkv: int, P2: int, page: int, head: int):
    b = C.c_int(0)
    off = lib().tkvo_record_offset(Hkv, P2, page, head, C.byref(b))
    return int(off), int(b.value)


def kcode_pos(bits, t, c):
    w, s = C.c_int(0), C.c_int(0)
    lib().tkvo_kcode_pos(C.c_int(bits), C.c_int(t), C.c_int(c), C.byref(w), C.byref(s))
    return int(w.value), int(s.value)


def vcode_pos(bits, t, c):
    w, s = C.c_int(0), C.c_int(0)
    lib().tkvo_vcode_pos(C.c_int(bits), C.c_int(t), C.c_int(c), C.byref(w), C.byref(s))
    return int(w.value), int(s.value)


def kmeta_index(t, g):
    return int(lib().tkvo_kmeta_index(C.c_int(t), C.c_int(g)))


def vmeta_index(t, g):
    return int(lib().tkvo_vmeta_index(C.c_int(t), C.c_int(g)))


def pack_pool(pool_u8, bit_map_u8, Hkv, P2, P4, slot_ids, bits, Kq, Vq):
    """Scatter canonical arrays into `pool` (modified in place)."""
    assert pool_u8.dtype == np.uint8 and pool_u8.flags.c_contiguous
    assert bit_map_u8.dtype == np.uint8 and bit_map_u8.flags.c_contiguous
    sl = _c(slot_ids, np.int64)
    bits = _c(bits, np.uint8)
    Kc, Ks, Kz = (_c(Kq[0], np.uint8), _c(Kq[1], np.uint16), _c(Kq[2], np.uint16))
    Vc, Vs, Vz = (_c(Vq[0], np.uint8), _c(Vq[1], np.uint16), _c(Vq[2], np.uint16))
    assert Kc.shape[1] == Hkv and Kc.shape[2] == HD
    rc = lib().tkvo_pack_pool(_p(pool_u8), _p(bit_map_u8), C.c_int(Hkv), C.c_int64(P2), C.c_int64(P4),
                              _p(sl), _p(bits), C.c_int64(sl.size),
                              _p(Kc), _p(Ks), _p(Kz), _p(Vc), _p(Vs), _p(Vz))
    if rc:
        raise ValueError("oracle pack_pool: slot / bitwidth mismatch")


def unpack_pool(pool_u8, Hkv, P2, P4, slot_ids):
    """Gather (Kq, Vq) canonical triples of the listed slots out of a pool."""
    pool = _c(pool_u8, np.uint8)
    sl = _c(slot_ids, np.int64)
    T = sl.size
    Kc = np.empty((T, Hkv, HD), np.uint8)
    Vc = np.empty((T, Hkv, HD), np.uint8)
    Ks, Kz, Vs, Vz = (np.empty((T, Hkv, NG), np.uint16) for _ in range(4))
    rc = lib().tkvo_unpack_pool(_p(pool), C.c_int(Hkv), C.c_int64(P2), C.c_int64(P4), _p(sl), C.c_int64(T),
                                _p(Kc), _p(Ks), _p(Kz), _p(Vc), _p(Vs), _p(Vz))
    if rc:
        raise ValueError("oracle unpack_pool: bad slot id")
    return (Kc, Ks, Kz), (Vc, Vs, Vz)
