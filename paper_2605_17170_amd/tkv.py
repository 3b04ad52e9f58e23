"""ctypes binding of libtkv (include/tkv.h): same names, argument marshalling
only.  Device buffers are torch tensors (torch is used for device memory and
streams, nothing else); host arrays are numpy.  Every step of the path runs in
the library's HIP kernels -- there is no fallback: if the library has not been
built, importing a function here raises."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtkv.so")

TKV_OK = 0
TKV_ERR_INVALID_ARG = -1
TKV_ERR_BAD_BITS = -2
TKV_ERR_BAD_SHAPE = -3
TKV_ERR_PAGE_RANGE = -4
TKV_ERR_POOL_EXHAUSTED = -5
TKV_ERR_WORKSPACE_TOO_SMALL = -6
TKV_ERR_HIP = -7
TKV_ERR_CAPACITY = -8
TKV_STATUS_TAG_MISMATCH = 1
TKV_STATUS_BITMAP_MISMATCH = 2
TKV_STATUS_PAGE_RANGE = 4
TKV_STATUS_DST_RANGE = 8
TKV_STATUS_BLOCK_PARTIAL = 16
TKV_STATUS_SCALE_SATURATED = 32
TKV_STATUS_BAD_ITEM = 64
TKV_KEYS_PER_TOKEN = 0
TKV_KEYS_PER_CHANNEL = 1

PAGE_TOKENS = 64
HEAD_DIM = 128
GROUP_SIZE = 32

EXPORTS = [
    "tkv_strerror", "tkv_record_bytes", "tkv_page_bytes", "tkv_pool_bytes", "tkv_record_offset",
    "tkv_alloc_create", "tkv_alloc_destroy", "tkv_alloc_pages", "tkv_free_pages", "tkv_alloc_free_count",
    "tkv_seq_create", "tkv_seq_destroy", "tkv_seq_release", "tkv_seq_n_tokens", "tkv_seq_n_pages",
    "tkv_seq_page_ids", "tkv_route_residual", "tkv_plan_append_max_work", "tkv_plan_append", "tkv_quantize_append", "tkv_gather_dequant",
    "tkv_plan_decode_capacity", "tkv_plan_decode", "tkv_decode_workspace_bytes", "tkv_decode_attention",
    "tkv_decode_split", "tkv_decode_reduce", "tkv_decode_attention_static", "tkv_allocate_bits_greedy", "tkv_allocate_bits_exhaustive",
    "tkv_tag_tokens", "tkv_tags_to_bits", "tkv_tag_counts", "tkv_probe_stream_read",
    "tkv_probe_decode_reads", "tkv_probe_stream_mix",
]


class TkvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (%d)" % (where, strerror(status), status))


class tkv_desc(C.Structure):
    _fields_ = [("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("group_size", C.c_int32),
                ("page_tokens", C.c_int32), ("n_pages_int2", C.c_int32), ("n_pages_int4", C.c_int32),
                ("int2_key_axis", C.c_int32)]

    @classmethod
    def make(cls, n_kv_heads, n_pages_int2, n_pages_int4, head_dim=HEAD_DIM, group_size=GROUP_SIZE,
             page_tokens=PAGE_TOKENS, int2_key_axis=0):
        return cls(n_kv_heads, head_dim, group_size, page_tokens, n_pages_int2, n_pages_int4, int2_key_axis)


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libtkv.so is not built: run `python -m paper_2605_17170_amd.build` "
                               "(there is no CPU fallback)")
        L = C.CDLL(LIB_PATH)
        vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
        dp = C.POINTER(tkv_desc)
        L.tkv_strerror.restype = C.c_char_p
        L.tkv_strerror.argtypes = [C.c_int]
        L.tkv_record_bytes.restype = sz
        L.tkv_record_bytes.argtypes = [C.c_int]
        L.tkv_page_bytes.restype = sz
        L.tkv_page_bytes.argtypes = [dp, C.c_int]
        L.tkv_pool_bytes.restype = sz
        L.tkv_pool_bytes.argtypes = [dp]
        L.tkv_record_offset.restype = sz
        L.tkv_record_offset.argtypes = [dp, i32, i32]
        L.tkv_alloc_create.argtypes = [dp, C.c_uint64, C.POINTER(vp)]
        L.tkv_alloc_destroy.restype = None
        L.tkv_alloc_destroy.argtypes = [vp]
        L.tkv_alloc_pages.argtypes = [vp, C.c_int, i32, vp]
        L.tkv_free_pages.argtypes = [vp, vp, i32]
        L.tkv_alloc_free_count.restype = i32
        L.tkv_alloc_free_count.argtypes = [vp, C.c_int]
        L.tkv_seq_create.argtypes = [C.POINTER(vp)]
        L.tkv_seq_destroy.restype = None
        L.tkv_seq_destroy.argtypes = [vp]
        L.tkv_seq_release.argtypes = [vp, vp]
        L.tkv_seq_n_tokens.restype = i32
        L.tkv_seq_n_tokens.argtypes = [vp, C.c_int]
        L.tkv_seq_n_pages.restype = i32
        L.tkv_seq_n_pages.argtypes = [vp, C.c_int]
        L.tkv_seq_page_ids.restype = i32
        L.tkv_seq_page_ids.argtypes = [vp, vp, i32]
        L.tkv_plan_append_max_work.restype = i32
        L.tkv_plan_append_max_work.argtypes = [i32]
        L.tkv_route_residual.restype = C.c_int
        L.tkv_route_residual.argtypes = [vp, i32, vp]
        L.tkv_plan_append.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp, i32, C.POINTER(i32)]
        L.tkv_quantize_append.argtypes = [dp, vp, vp, vp, vp, vp, i32, i32, vp, vp, i32, vp, vp]
        L.tkv_gather_dequant.restype = C.c_int
        L.tkv_gather_dequant.argtypes = [dp, vp, vp, vp, vp, i32, vp, vp, i32, vp, vp]
        L.tkv_plan_decode_capacity.restype = i32
        L.tkv_plan_decode_capacity.argtypes = [i32, i32]
        L.tkv_plan_decode.restype = i32
        L.tkv_plan_decode.argtypes = [dp, i32, vp, vp, vp, i32, vp, i32, vp]
        L.tkv_decode_workspace_bytes.restype = sz
        L.tkv_decode_workspace_bytes.argtypes = [dp, i32, i32]
        L.tkv_decode_attention.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, C.c_float,
                                           vp, vp, sz, vp, vp]
        L.tkv_decode_attention_static.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, C.c_float,
                                                  vp, vp, vp]
        L.tkv_decode_split.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, C.c_float, vp, sz, vp, vp]
        L.tkv_decode_reduce.argtypes = [dp, vp, i32, i32, i32, vp, vp, sz, vp]
        L.tkv_probe_stream_read.argtypes = [vp, sz, vp, vp]
        L.tkv_probe_decode_reads.argtypes = [dp, vp, vp, vp, vp, vp, vp, i32, i32, i32, vp, vp]
        L.tkv_probe_stream_mix.argtypes = [vp, vp, sz, i32, i32, vp]
        L.tkv_tag_tokens.argtypes = [vp, vp, i32, vp]
        L.tkv_tags_to_bits.argtypes = [vp, i32, vp, vp]
        L.tkv_tag_counts.argtypes = [vp, i32, vp]
        for fn in (L.tkv_allocate_bits_greedy, L.tkv_allocate_bits_exhaustive):
            fn.restype = C.c_int
            fn.argtypes = [i32, C.POINTER(C.c_int64), C.POINTER(C.c_double), C.POINTER(C.c_double), C.c_double,
                           C.POINTER(C.c_uint8)]
        _lib = L
    return _lib


def strerror(status: int) -> str:
    return lib().tkv_strerror(status).decode()


def _check(status: int, where: str):
    if status < 0:
        raise TkvError(status, where)
    return status


def _np(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a, C.c_void_p(a.ctypes.data if a.size else None)


def _dev(t):
    """Device pointer of a torch tensor (None -> NULL)."""
    if t is None:
        return C.c_void_p(None)
    assert t.is_contiguous(), "device arguments must be contiguous"
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return C.c_void_p(getattr(stream, "cuda_stream", stream))


class Prepared:
    """One call of an entry point with its arguments marshalled once.  Loops that repeat the same call on the same
    buffers and stream (a decode step per layer, a benchmark) pay for building the ctypes arguments only the first
    time: `call = tkv_decode_attention(..., prepare=True)`, then `call()`.  The tensors are kept alive here."""
    __slots__ = ("fn", "cargs", "where", "keep")

    def __init__(self, fn, cargs, where, keep):
        self.fn, self.cargs, self.where, self.keep = fn, cargs, where, keep

    def __call__(self):
        st = self.fn(*self.cargs)
        if st < 0:
            _check(st, self.where)


def _run(fn, cargs, where, keep, prepare):
    call = Prepared(fn, cargs, where, keep)
    if prepare:
        return call
    call()


# ---------------------------------------------------------------- geometry
def tkv_record_bytes(bits: int) -> int:
    return int(lib().tkv_record_bytes(bits))


def tkv_page_bytes(desc: tkv_desc, bits: int) -> int:
    return int(lib().tkv_page_bytes(C.byref(desc), bits))


def tkv_pool_bytes(desc: tkv_desc) -> int:
    return int(lib().tkv_pool_bytes(C.byref(desc)))


def tkv_record_offset(desc: tkv_desc, page: int, head: int) -> int:
    v = int(lib().tkv_record_offset(C.byref(desc), page, head))
    return -1 if v == C.c_size_t(-1).value else v


# ---------------------------------------------------------------- allocator / sequences (host)
def tkv_alloc_create(desc: tkv_desc, shuffle_seed: int = 0):
    h = C.c_void_p()
    _check(lib().tkv_alloc_create(C.byref(desc), shuffle_seed, C.byref(h)), "tkv_alloc_create")
    return h


def tkv_alloc_destroy(a):
    lib().tkv_alloc_destroy(a)


def tkv_alloc_pages(a, bits: int, n: int) -> np.ndarray:
    out = np.empty(max(n, 0), np.int32)
    _check(lib().tkv_alloc_pages(a, bits, n, C.c_void_p(out.ctypes.data if n > 0 else None)), "tkv_alloc_pages")
    return out


def tkv_free_pages(a, page_ids):
    ids, p = _np(page_ids, np.int32)
    _check(lib().tkv_free_pages(a, p, ids.size), "tkv_free_pages")


def tkv_alloc_free_count(a, bits: int) -> int:
    return _check(lib().tkv_alloc_free_count(a, bits), "tkv_alloc_free_count")


def tkv_seq_create():
    h = C.c_void_p()
    _check(lib().tkv_seq_create(C.byref(h)), "tkv_seq_create")
    return h


def tkv_seq_destroy(s):
    lib().tkv_seq_destroy(s)


def tkv_seq_release(s, a):
    _check(lib().tkv_seq_release(s, a), "tkv_seq_release")


def tkv_seq_n_tokens(s, bits: int) -> int:
    return _check(lib().tkv_seq_n_tokens(s, bits), "tkv_seq_n_tokens")


def tkv_seq_n_pages(s, bits: int) -> int:
    return _check(lib().tkv_seq_n_pages(s, bits), "tkv_seq_n_pages")


def tkv_seq_page_ids(s) -> np.ndarray:
    n = tkv_seq_n_pages(s, 2) + tkv_seq_n_pages(s, 4)
    out = np.empty(n, np.int32)
    got = _check(lib().tkv_seq_page_ids(s, C.c_void_p(out.ctypes.data if n else None), n), "tkv_seq_page_ids")
    assert got == n
    return out


# ---------------------------------------------------------------- Q1 (host)
def tkv_route_residual(tag_bits) -> np.ndarray:
    """Per-token widths after the residual policy of per-channel INT2 keys (u8[n])."""
    bits, pb = _np(tag_bits, np.uint8)
    out = np.empty(bits.size, np.uint8)
    _check(lib().tkv_route_residual(pb, bits.size, C.c_void_p(out.ctypes.data if bits.size else None)),
           "tkv_route_residual")
    return out


def tkv_plan_append_max_work(n_tokens: int) -> int:
    return _check(lib().tkv_plan_append_max_work(n_tokens), "tkv_plan_append_max_work")


def tkv_plan_append(a, s, tag_bits, token_base: int = 0):
    """Returns (slot_ids i32[n], work_pages i32[n_work], work_src i32[n_work, 64])."""
    bits, pb = _np(tag_bits, np.uint8)
    n = bits.size
    cap = tkv_plan_append_max_work(n)
    slots = np.empty(n, np.int32)
    wp = np.empty(cap, np.int32)
    ws = np.empty((cap, PAGE_TOKENS), np.int32)
    nw = C.c_int32(0)
    _check(lib().tkv_plan_append(a, s, pb, n, token_base, C.c_void_p(slots.ctypes.data if n else None),
                                 C.c_void_p(wp.ctypes.data), C.c_void_p(ws.ctypes.data), cap, C.byref(nw)),
           "tkv_plan_append")
    return slots, wp[:nw.value].copy(), ws[:nw.value].copy()


# ---------------------------------------------------------------- Q2-Q5 (device)
def tkv_quantize_append(desc, pool, bit_map, K, V, tag_bits, work_pages, work_src, status=None, stream=None,
                        group_size: int = GROUP_SIZE, prepare=False):
    """All array arguments are torch device tensors: pool u8, bit_map u8,
    K/V bf16 [T,Hkv,D], tag_bits u8[T], work_pages i32[n_work], work_src i32[n_work,64]."""
    n_tokens = int(K.shape[0]) if K is not None else 0
    n_work = int(work_pages.numel()) if work_pages is not None else 0
    if K is not None:
        assert tuple(V.shape) == tuple(K.shape) == (n_tokens, desc.n_kv_heads, desc.head_dim)
        assert K.element_size() == 2 and V.element_size() == 2 and tag_bits.numel() == n_tokens
    if n_work:
        assert work_src.numel() == n_work * desc.page_tokens and work_src.element_size() == 4
        assert pool.numel() * pool.element_size() >= tkv_pool_bytes(desc)
        assert bit_map.numel() >= desc.n_pages_int2 + desc.n_pages_int4
    return _run(lib().tkv_quantize_append,
                (C.byref(desc), _dev(pool), _dev(bit_map), _dev(K), _dev(V), _dev(tag_bits), n_tokens, group_size,
                 _dev(work_pages), _dev(work_src), n_work, _dev(status), _stream(stream)),
                "tkv_quantize_append", (desc, pool, bit_map, K, V, tag_bits, work_pages, work_src, status, stream), prepare)


# ---------------------------------------------------------------- P1 (device)
def tkv_gather_dequant(desc, pool, bit_map, work_pages, work_dst, K_out, V_out, status=None, stream=None):
    """Prefill gather: pool u8, bit_map u8, work_pages i32[n_work], work_dst i32[n_work,64] (output row per
    slot or -1), K_out/V_out fp16 [T,Hkv,D]; all torch device tensors."""
    n_work = int(work_pages.numel()) if work_pages is not None else 0
    n_tokens = int(K_out.shape[0]) if K_out is not None else 0
    if n_work:
        assert tuple(V_out.shape) == tuple(K_out.shape) == (n_tokens, desc.n_kv_heads, desc.head_dim)
        assert K_out.element_size() == 2 and V_out.element_size() == 2
        assert K_out.is_contiguous() and V_out.is_contiguous()
        assert work_dst.numel() == n_work * desc.page_tokens and work_dst.element_size() == 4
        assert pool.numel() * pool.element_size() >= tkv_pool_bytes(desc)
        assert bit_map.numel() >= desc.n_pages_int2 + desc.n_pages_int4
    _check(lib().tkv_gather_dequant(C.byref(desc), _dev(pool), _dev(bit_map), _dev(work_pages), _dev(work_dst), n_work,
                                    _dev(K_out), _dev(V_out), n_tokens, _dev(status), _stream(stream)),
           "tkv_gather_dequant")


# ---------------------------------------------------------------- D1 (host)
def tkv_plan_decode_capacity(batch: int, target_items: int) -> int:
    return _check(lib().tkv_plan_decode_capacity(batch, target_items), "tkv_plan_decode_capacity")


def tkv_plan_decode(desc, page_indptr, n_tok_int2, n_tok_int4, target_items: int):
    """Returns (items i32[n_items, 4], seq_item_indptr i32[batch+1])."""
    ip, pip = _np(page_indptr, np.int32)
    n2, p2 = _np(n_tok_int2, np.int32)
    n4, p4 = _np(n_tok_int4, np.int32)
    batch = ip.size - 1
    cap = tkv_plan_decode_capacity(batch, target_items)
    items = np.empty((cap, 4), np.int32)
    sip = np.empty(batch + 1, np.int32)
    n = _check(lib().tkv_plan_decode(C.byref(desc), batch, pip, p2, p4, target_items,
                                     C.c_void_p(items.ctypes.data), cap, C.c_void_p(sip.ctypes.data)),
               "tkv_plan_decode")
    return items[:n].copy(), sip


# ---------------------------------------------------------------- D2-D7 (device)
def tkv_decode_workspace_bytes(desc, n_items: int, n_q_heads: int) -> int:
    return int(lib().tkv_decode_workspace_bytes(C.byref(desc), n_items, n_q_heads))


def tkv_decode_attention(desc, pool, bit_map, q, page_indptr, page_ids, n_tok_int2, n_tok_int4, items,
                         seq_item_indptr, sm_scale: float, out, workspace, status=None, stream=None, prepare=False):
    """Device tensors: q bf16 [B,Hq,D]; page_indptr i32[B+1]; page_ids i32; n_tok_int2/4 i32[B];
    items i32[n_items,4]; seq_item_indptr i32[B+1]; out f32 [B,Hq,D]; workspace u8."""
    batch, n_q_heads = int(q.shape[0]), int(q.shape[1])
    n_items = int(items.shape[0]) if items is not None else 0
    ws_bytes = int(workspace.numel() * workspace.element_size()) if workspace is not None else 0
    assert q.element_size() == 2 and int(q.shape[2]) == desc.head_dim
    assert page_indptr.numel() == batch + 1 and seq_item_indptr.numel() == batch + 1
    assert n_tok_int2.numel() == batch and n_tok_int4.numel() == batch
    assert out.numel() == batch * n_q_heads * desc.head_dim and out.element_size() == 4
    if n_items:
        assert items.numel() == 4 * n_items and pool.numel() * pool.element_size() >= tkv_pool_bytes(desc)
    return _run(lib().tkv_decode_attention,
                (C.byref(desc), _dev(pool), _dev(bit_map), _dev(q), _dev(page_indptr), _dev(page_ids), _dev(n_tok_int2),
                 _dev(n_tok_int4), _dev(items), _dev(seq_item_indptr), n_items, batch, n_q_heads, float(sm_scale),
                 _dev(out), _dev(workspace), ws_bytes, _dev(status), _stream(stream)),
                "tkv_decode_attention",
                (desc, pool, bit_map, q, page_indptr, page_ids, n_tok_int2, n_tok_int4, items, seq_item_indptr, out, workspace,
                 status, stream), prepare)


TKV_DECODE_STATIC_SCRATCH_BYTES = 16 << 20


def tkv_decode_attention_static(desc, pool, bit_map, q, page_indptr, page_ids, n_tok_int2, n_tok_int4, items,
                                seq_item_indptr, sm_scale: float, out, status=None, stream=None):
    """tkv_decode_attention with the partials in the library's fixed device array (no workspace argument,
    nothing allocated); same device tensors otherwise."""
    batch, n_q_heads = int(q.shape[0]), int(q.shape[1])
    n_items = int(items.shape[0]) if items is not None else 0
    assert q.element_size() == 2 and int(q.shape[2]) == desc.head_dim
    assert page_indptr.numel() == batch + 1 and seq_item_indptr.numel() == batch + 1
    assert n_tok_int2.numel() == batch and n_tok_int4.numel() == batch
    assert out.numel() == batch * n_q_heads * desc.head_dim and out.element_size() == 4
    if n_items:
        assert items.numel() == 4 * n_items and pool.numel() * pool.element_size() >= tkv_pool_bytes(desc)
    _check(lib().tkv_decode_attention_static(C.byref(desc), _dev(pool), _dev(bit_map), _dev(q), _dev(page_indptr),
                                             _dev(page_ids), _dev(n_tok_int2), _dev(n_tok_int4), _dev(items),
                                             _dev(seq_item_indptr), n_items, batch, n_q_heads, float(sm_scale),
                                             _dev(out), _dev(status), _stream(stream)),
           "tkv_decode_attention_static")


def tkv_decode_split(desc, pool, bit_map, q, page_indptr, page_ids, n_tok_int2, n_tok_int4, items, sm_scale: float,
                     workspace, status=None, stream=None, prepare=False):
    """D2-D6 only: leaves the per-item partials in `workspace`."""
    batch, n_q_heads = int(q.shape[0]), int(q.shape[1])
    n_items = int(items.shape[0]) if items is not None else 0
    ws_bytes = int(workspace.numel() * workspace.element_size()) if workspace is not None else 0
    assert q.element_size() == 2 and int(q.shape[2]) == desc.head_dim and page_indptr.numel() == batch + 1
    assert n_tok_int2.numel() == batch and n_tok_int4.numel() == batch
    if n_items:
        assert items.numel() == 4 * n_items and pool.numel() * pool.element_size() >= tkv_pool_bytes(desc)
    return _run(lib().tkv_decode_split,
                (C.byref(desc), _dev(pool), _dev(bit_map), _dev(q), _dev(page_indptr), _dev(page_ids), _dev(n_tok_int2),
                 _dev(n_tok_int4), _dev(items), n_items, batch, n_q_heads, float(sm_scale), _dev(workspace), ws_bytes,
                 _dev(status), _stream(stream)),
                "tkv_decode_split",
                (desc, pool, bit_map, q, page_indptr, page_ids, n_tok_int2, n_tok_int4, items, workspace, status, stream), prepare)


def tkv_decode_reduce(desc, seq_item_indptr, n_items: int, out, workspace, stream=None):
    """D7 only: merges the partials in `workspace` into out f32 [B,Hq,D]."""
    batch, n_q_heads = int(out.shape[0]), int(out.shape[1])
    ws_bytes = int(workspace.numel() * workspace.element_size()) if workspace is not None else 0
    assert seq_item_indptr.numel() == batch + 1 and out.element_size() == 4
    _check(lib().tkv_decode_reduce(C.byref(desc), _dev(seq_item_indptr), n_items, batch, n_q_heads, _dev(out),
                                   _dev(workspace), ws_bytes, _stream(stream)), "tkv_decode_reduce")


def _allocate_bits(fn, name, N, D2, D4, B):
    n = len(N)
    if not (len(D2) == n and len(D4) == n):
        raise ValueError("N, D2 and D4 must have one entry per tag")
    out = (C.c_uint8 * n)()
    _check(fn(n, (C.c_int64 * n)(*[int(x) for x in N]), (C.c_double * n)(*[float(x) for x in D2]),
              (C.c_double * n)(*[float(x) for x in D4]), float(B), out), name)
    return list(out)


def tkv_allocate_bits_greedy(N, D2, D4, B):
    """Tag bitwidths (2 or 4) by the greedy walk over per-bit gains; argument marshalling only."""
    return _allocate_bits(lib().tkv_allocate_bits_greedy, "tkv_allocate_bits_greedy", N, D2, D4, B)


def tkv_allocate_bits_exhaustive(N, D2, D4, B):
    """Tag bitwidths (2 or 4) by exhaustive search, at most 22 tags; argument marshalling only."""
    return _allocate_bits(lib().tkv_allocate_bits_exhaustive, "tkv_allocate_bits_exhaustive", N, D2, D4, B)


# ---------------------------------------------------------------- T1 (host)
N_TAGS = 56


def tkv_tag_tokens(semantic, modal) -> np.ndarray:
    """Tag codes u8[n] from per-token semantic role and modality (u8[n] each)."""
    sem, ps = _np(semantic, np.uint8)
    mod, pm = _np(modal, np.uint8)
    if sem.shape != mod.shape:
        raise ValueError("semantic and modal must have one entry per token")
    out = np.empty(sem.size, np.uint8)
    _check(lib().tkv_tag_tokens(ps, pm, sem.size, C.c_void_p(out.ctypes.data if sem.size else None)), "tkv_tag_tokens")
    return out


def tkv_tags_to_bits(tags, table) -> np.ndarray:
    tg, pt = _np(tags, np.uint8)
    tb, pb = _np(table, np.uint8)
    if tb.size != N_TAGS:
        raise ValueError("the table has one entry per tag (56)")
    out = np.empty(tg.size, np.uint8)
    _check(lib().tkv_tags_to_bits(pt, tg.size, pb, C.c_void_p(out.ctypes.data if tg.size else None)), "tkv_tags_to_bits")
    return out


def tkv_tag_counts(tags) -> np.ndarray:
    tg, pt = _np(tags, np.uint8)
    counts = np.zeros(N_TAGS, np.int64)
    _check(lib().tkv_tag_counts(pt, tg.size, C.c_void_p(counts.ctypes.data)), "tkv_tag_counts")
    return counts


# ---------------------------------------------------------------- measurement aid (device)
def tkv_probe_stream_read(buf, stream=None):
    """Plain 128-bit streaming read of a torch device tensor (read-bandwidth ceiling for benchmarks)."""
    nbytes = buf.numel() * buf.element_size()
    _check(lib().tkv_probe_stream_read(_dev(buf), nbytes - nbytes % 16, C.c_void_p(None), _stream(stream)),
           "tkv_probe_stream_read")


def tkv_probe_decode_reads(desc, pool, page_indptr, page_ids, n_tok_int2, n_tok_int4, items, batch: int, walk: bool,
                           stream=None, prepare=False):
    """The record reads of a decode plan without the arithmetic (device tensors as for tkv_decode_split)."""
    n_items = int(items.shape[0]) if items is not None else 0
    return _run(lib().tkv_probe_decode_reads,
                (C.byref(desc), _dev(pool), _dev(page_indptr), _dev(page_ids), _dev(n_tok_int2), _dev(n_tok_int4), _dev(items),
                 n_items, batch, 1 if walk else 0, C.c_void_p(None), _stream(stream)),
                "tkv_probe_decode_reads", (desc, pool, page_indptr, page_ids, n_tok_int2, n_tok_int4, items, stream), prepare)


def tkv_probe_stream_mix(src, dst, unit_bytes: int, read_parts: int, write_parts: int, stream=None, prepare=False):
    """Streaming read of read_parts * unit_bytes of `src` and write of write_parts * unit_bytes of `dst`."""
    assert src.numel() * src.element_size() >= read_parts * unit_bytes
    assert dst.numel() * dst.element_size() >= write_parts * unit_bytes
    return _run(lib().tkv_probe_stream_mix, (_dev(src), _dev(dst), unit_bytes, read_parts, write_parts, _stream(stream)),
                "tkv_probe_stream_mix", (src, dst, stream), prepare)
