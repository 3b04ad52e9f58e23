"""CPU-only tests of libtkv's host side: the library loads and exports every
symbol the header declares, geometry agrees with the oracle's codec, the
allocators / sequence tables / planners keep their invariants, and every
argument error is reported before anything is launched (so these run
without a GPU)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2605_17170_amd import tkv

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "tkv.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(tkv_[a-z0-9_]+)\s*\(", hdr))
    assert declared == set(tkv.EXPORTS)
    L = tkv.lib()
    for name in declared:
        assert getattr(L, name) is not None


def test_geometry_matches_oracle_codec(oracle):
    d = tkv.tkv_desc.make(8, 10, 20)
    assert tkv.tkv_record_bytes(2) == oracle.record_bytes(2) == 6144
    assert tkv.tkv_record_bytes(4) == oracle.record_bytes(4) == 10240
    assert tkv.tkv_record_bytes(3) == 0
    assert tkv.tkv_pool_bytes(d) == oracle.pool_bytes(8, 10, 20)
    assert tkv.tkv_page_bytes(d, 2) == 8 * 6144 and tkv.tkv_page_bytes(d, 4) == 8 * 10240
    for page, head in [(0, 0), (3, 5), (9, 7), (10, 0), (12, 1), (29, 7)]:
        assert tkv.tkv_record_offset(d, page, head) == oracle.record_offset(8, 10, page, head)[0]
    assert tkv.tkv_record_offset(d, 30, 0) == -1 and tkv.tkv_record_offset(d, 0, 8) == -1
    bad = tkv.tkv_desc.make(8, 10, 20, head_dim=64)
    assert tkv.tkv_pool_bytes(bad) == 0


def test_allocator_pools_are_independent():
    d = tkv.tkv_desc.make(2, 5, 3)
    a = tkv.tkv_alloc_create(d, 0)
    assert tkv.tkv_alloc_free_count(a, 2) == 5 and tkv.tkv_alloc_free_count(a, 4) == 3
    p2 = tkv.tkv_alloc_pages(a, 2, 3)
    p4 = tkv.tkv_alloc_pages(a, 4, 3)
    assert p2.tolist() == [0, 1, 2] and p4.tolist() == [5, 6, 7]      # in-order without a seed
    assert tkv.tkv_alloc_free_count(a, 2) == 2 and tkv.tkv_alloc_free_count(a, 4) == 0
    with pytest.raises(tkv.TkvError) as e:
        tkv.tkv_alloc_pages(a, 4, 1)
    assert e.value.status == tkv.TKV_ERR_POOL_EXHAUSTED
    with pytest.raises(tkv.TkvError) as e:
        tkv.tkv_alloc_pages(a, 2, 3)                                   # only 2 left: nothing taken
    assert e.value.status == tkv.TKV_ERR_POOL_EXHAUSTED and tkv.tkv_alloc_free_count(a, 2) == 2
    with pytest.raises(tkv.TkvError) as e:
        tkv.tkv_alloc_pages(a, 3, 1)
    assert e.value.status == tkv.TKV_ERR_BAD_BITS
    tkv.tkv_free_pages(a, [6, 1])
    assert tkv.tkv_alloc_free_count(a, 2) == 3 and tkv.tkv_alloc_free_count(a, 4) == 1
    for ids in ([1], [8], [-1], [0, 0]):                               # double free, range, duplicate
        with pytest.raises(tkv.TkvError) as e:
            tkv.tkv_free_pages(a, ids)
        assert e.value.status == tkv.TKV_ERR_PAGE_RANGE
    assert tkv.tkv_alloc_free_count(a, 2) == 3                         # failed frees change nothing
    tkv.tkv_alloc_destroy(a)


def test_shuffled_allocator_is_a_seeded_permutation():
    d = tkv.tkv_desc.make(1, 200, 100)
    out = []
    for seed in (7, 7, 8):
        a = tkv.tkv_alloc_create(d, seed)
        out.append((tkv.tkv_alloc_pages(a, 2, 200), tkv.tkv_alloc_pages(a, 4, 100)))
        tkv.tkv_alloc_destroy(a)
    assert sorted(out[0][0]) == list(range(200)) and sorted(out[0][1]) == list(range(200, 300))
    assert np.array_equal(out[0][0], out[1][0]) and not np.array_equal(out[0][0], out[2][0])
    assert not np.array_equal(out[0][0], np.arange(200))


def _check_plan(bits, slots, wp, ws, page_list_2, page_list_4, start2, start4, base, P2):
    """Invariants of an append plan."""
    # tokens of each width fill that width's page stream in arrival order
    for b, pages, start in ((2, page_list_2, start2), (4, page_list_4, start4)):
        idx = np.nonzero(bits == b)[0]
        pos = start + np.arange(idx.size)
        want = np.asarray(pages, np.int64)[pos // 64] * 64 + pos % 64 if idx.size else np.zeros(0, np.int64)
        assert np.array_equal(slots[idx], want)
    assert np.unique(slots).size == slots.size
    # every token's page is in its own pool
    assert np.all((slots // 64 < P2) == (bits == 2))
    # the gather list is the inverse of slot_ids
    assert np.unique(wp).size == wp.size
    want_src = {int(s): base + t for t, s in enumerate(slots)}
    got_src = {}
    for w, page in enumerate(wp):
        for s in range(64):
            if ws[w, s] >= 0:
                got_src[int(page) * 64 + s] = int(ws[w, s])
    assert got_src == want_src


def test_plan_append_routes_tokens_and_grows_page_tables():
    rng = np.random.default_rng(0)
    d = tkv.tkv_desc.make(2, 40, 40)
    a = tkv.tkv_alloc_create(d, 5)
    s = tkv.tkv_seq_create()
    n2 = n4 = 0
    for step, n in enumerate([100, 1, 63, 0, 200, 7]):
        bits = rng.choice([2, 4], n).astype(np.uint8)
        slots, wp, ws = tkv.tkv_plan_append(a, s, bits, token_base=1000 * step)
        pages = tkv.tkv_seq_page_ids(s)
        np2, np4 = tkv.tkv_seq_n_pages(s, 2), tkv.tkv_seq_n_pages(s, 4)
        assert pages.size == np2 + np4 and np.all(pages[:np2] < 40) and np.all(pages[np2:] >= 40)
        _check_plan(bits, slots, wp, ws, pages[:np2], pages[np2:], n2, n4, 1000 * step, 40)
        n2 += int((bits == 2).sum()); n4 += int((bits == 4).sum())
        assert tkv.tkv_seq_n_tokens(s, 2) == n2 and tkv.tkv_seq_n_tokens(s, 4) == n4
        assert np2 == -(-n2 // 64) and np4 == -(-n4 // 64)
        assert wp.size <= tkv.tkv_plan_append_max_work(n)
    used = 80 - tkv.tkv_alloc_free_count(a, 2) - tkv.tkv_alloc_free_count(a, 4)
    assert used == tkv.tkv_seq_n_pages(s, 2) + tkv.tkv_seq_n_pages(s, 4)
    tkv.tkv_seq_release(s, a)
    assert tkv.tkv_alloc_free_count(a, 2) == 40 and tkv.tkv_alloc_free_count(a, 4) == 40
    assert tkv.tkv_seq_n_tokens(s, 2) == 0 and tkv.tkv_seq_page_ids(s).size == 0
    tkv.tkv_seq_destroy(s)
    tkv.tkv_alloc_destroy(a)


def test_plan_append_errors_leave_state_unchanged():
    d = tkv.tkv_desc.make(1, 2, 2)
    a = tkv.tkv_alloc_create(d, 0)
    s = tkv.tkv_seq_create()
    with pytest.raises(tkv.TkvError) as e:
        tkv.tkv_plan_append(a, s, np.uint8([2, 4, 3]))
    assert e.value.status == tkv.TKV_ERR_BAD_BITS
    with pytest.raises(tkv.TkvError) as e:
        tkv.tkv_plan_append(a, s, np.uint8([2] * 10 + [4] * 129))     # needs 3 INT4 pages, 2 exist
    assert e.value.status == tkv.TKV_ERR_POOL_EXHAUSTED
    assert tkv.tkv_alloc_free_count(a, 2) == 2 and tkv.tkv_alloc_free_count(a, 4) == 2
    assert tkv.tkv_seq_n_tokens(s, 2) == 0 and tkv.tkv_seq_n_pages(s, 4) == 0
    slots, wp, ws = tkv.tkv_plan_append(a, s, np.uint8([2] * 128 + [4] * 128))
    assert tkv.tkv_alloc_free_count(a, 2) == 0 and wp.size == 4
    tkv.tkv_seq_destroy(s)
    tkv.tkv_alloc_destroy(a)


@pytest.mark.parametrize("target", [1, 7, 64, 1000])
def test_plan_decode_covers_every_page_once_and_balances_bytes(target):
    rng = np.random.default_rng(target)
    d = tkv.tkv_desc.make(8, 4096, 4096)
    B = 9
    n2 = rng.integers(0, 9000, B).astype(np.int32)
    n4 = rng.integers(0, 4000, B).astype(np.int32)
    n2[2] = n4[2] = 0                 # an empty sequence
    n4[3] = 0                         # INT2 only
    n2[4] = 0                         # INT4 only
    n2[5], n4[5] = 1, 1               # two one-token pages
    pages = -(-n2 // 64) + -(-n4 // 64)
    ip = np.concatenate([[0], np.cumsum(pages)]).astype(np.int32)
    items, sip = tkv.tkv_plan_decode(d, ip, n2, n4, target)
    assert sip[0] == 0 and sip[-1] == items.shape[0] and np.all(np.diff(sip) >= 0)
    # items come in launch order; their partial slots are a permutation in sequence order
    assert sorted(items[:, 3].tolist()) == list(range(items.shape[0]))
    p2_of = -(-n2 // 64)
    share2 = np.array([(min(hi, p2_of[b]) - min(lo, p2_of[b])) * 4096 // (hi - lo) for b, lo, hi, _ in items])
    assert np.all(np.diff(share2) <= 0), "launch order: falling share of INT2 pages"
    items = items[np.argsort(items[:, 3])]
    assert items.shape[0] <= tkv.tkv_plan_decode_capacity(B, target)
    cost = lambda b, lo, hi: 6 * (min(hi, -(-n2[b] // 64)) - min(lo, -(-n2[b] // 64))) + \
        7 * (max(hi, -(-n2[b] // 64)) - max(lo, -(-n2[b] // 64)))
    costs = []
    for b in range(B):
        its = items[sip[b]:sip[b + 1]]
        assert np.all(its[:, 0] == b)
        if pages[b] == 0:
            assert its.shape[0] == 0
            continue
        assert its[0, 1] == 0 and its[-1, 2] == pages[b]
        assert np.all(its[1:, 1] == its[:-1, 2]) and np.all(its[:, 2] > its[:, 1])
        costs += [cost(b, lo, hi) for _, lo, hi, _ in its]
    total = sum(6 * -(-int(a) // 64) + 7 * -(-int(b) // 64) for a, b in zip(n2, n4))
    assert sum(costs) == total
    if target >= 64:
        per = total / target
        assert max(costs) <= 2.0 * per + 10       # no item much heavier than the target share
    if target == 64:
        assert abs(items.shape[0] - target) <= B + 1


def test_plan_decode_rejects_inconsistent_page_table():
    d = tkv.tkv_desc.make(1, 10, 10)
    with pytest.raises(tkv.TkvError) as e:
        tkv.tkv_plan_decode(d, np.int32([0, 3]), np.int32([64]), np.int32([64]), 4)   # 2 pages, table says 3
    assert e.value.status == tkv.TKV_ERR_INVALID_ARG


def test_device_entry_points_validate_before_launch():
    """No GPU here: every call must return its error without touching HIP."""
    L = tkv.lib()
    d = tkv.tkv_desc.make(8, 4, 4)
    fake = C.c_void_p(0x1000)   # 256-aligned non-null stand-in; never dereferenced on these paths
    null = C.c_void_p(None)
    byref = C.byref
    # append
    assert L.tkv_quantize_append(None, fake, fake, fake, fake, fake, 1, 32, fake, fake, 1, null, null) == tkv.TKV_ERR_INVALID_ARG
    assert L.tkv_quantize_append(byref(tkv.tkv_desc.make(8, 4, 4, head_dim=64)), fake, fake, fake, fake, fake, 1, 32, fake, fake, 1, null, null) == tkv.TKV_ERR_BAD_SHAPE
    assert L.tkv_quantize_append(byref(d), fake, fake, fake, fake, fake, 1, 64, fake, fake, 1, null, null) == tkv.TKV_ERR_BAD_SHAPE
    assert L.tkv_quantize_append(byref(d), fake, fake, fake, fake, fake, 1, 32, fake, fake, -1, null, null) == tkv.TKV_ERR_INVALID_ARG
    assert L.tkv_quantize_append(byref(d), null, fake, fake, fake, fake, 1, 32, fake, fake, 1, null, null) == tkv.TKV_ERR_INVALID_ARG
    assert L.tkv_quantize_append(byref(d), C.c_void_p(0x1010), fake, fake, fake, fake, 1, 32, fake, fake, 1, null, null) == tkv.TKV_ERR_INVALID_ARG
    assert L.tkv_quantize_append(byref(d), fake, fake, fake, fake, fake, 1, 32, fake, fake, 0, null, null) == tkv.TKV_OK   # nothing to do
    # decode
    args = dict(pool=fake, bm=fake, q=fake, ip=fake, ids=fake, n2=fake, n4=fake, items=fake, sip=fake,
                n_items=4, batch=2, hq=64, sm=C.c_float(0.088), out=fake, ws=fake, wsb=C.c_size_t(1 << 30))

    def call(desc=d, **kw):
        a = dict(args, **kw)
        return L.tkv_decode_attention(byref(desc), a["pool"], a["bm"], a["q"], a["ip"], a["ids"], a["n2"], a["n4"],
                                      a["items"], a["sip"], a["n_items"], a["batch"], a["hq"], a["sm"], a["out"],
                                      a["ws"], a["wsb"], null, null)

    assert call(hq=60) == tkv.TKV_ERR_BAD_SHAPE                    # not a multiple of the kv heads
    assert call(hq=128) == tkv.TKV_ERR_BAD_SHAPE                   # 16 query heads per kv head
    assert call(hq=0) == tkv.TKV_ERR_INVALID_ARG
    assert call(q=null) == tkv.TKV_ERR_INVALID_ARG
    assert call(out=null) == tkv.TKV_ERR_INVALID_ARG
    assert call(ws=null) == tkv.TKV_ERR_INVALID_ARG
    assert call(sm=C.c_float(0.0)) == tkv.TKV_ERR_INVALID_ARG
    assert call(sm=C.c_float(float("nan"))) == tkv.TKV_ERR_INVALID_ARG
    need = tkv.tkv_decode_workspace_bytes(d, 4, 64)
    assert need == 4 * 64 * 130 * 4
    assert call(wsb=C.c_size_t(need - 1)) == tkv.TKV_ERR_WORKSPACE_TOO_SMALL
    assert call(batch=0) == tkv.TKV_OK
    assert tkv.strerror(tkv.TKV_ERR_WORKSPACE_TOO_SMALL) == "workspace too small"


def test_split_and_reduce_entry_points_validate_before_launch():
    L = tkv.lib()
    d = tkv.tkv_desc.make(8, 4, 4)
    fake, null = C.c_void_p(0x1000), C.c_void_p(None)
    big = C.c_size_t(1 << 30)
    sm = C.c_float(0.088)
    ok_args = [fake] * 9
    assert L.tkv_decode_split(C.byref(d), *ok_args[:8], 4, 2, 60, sm, fake, big, null, null) == tkv.TKV_ERR_BAD_SHAPE
    assert L.tkv_decode_split(C.byref(d), null, *ok_args[:7], 4, 2, 64, sm, fake, big, null, null) == tkv.TKV_ERR_INVALID_ARG
    assert L.tkv_decode_split(C.byref(d), *ok_args[:8], 4, 2, 64, sm, fake, C.c_size_t(16), null, null) == tkv.TKV_ERR_WORKSPACE_TOO_SMALL
    assert L.tkv_decode_split(C.byref(d), *ok_args[:8], 0, 2, 64, sm, fake, big, null, null) == tkv.TKV_OK   # no items: nothing to do
    assert L.tkv_decode_reduce(C.byref(d), fake, 4, 2, 64, null, fake, big, null) == tkv.TKV_ERR_INVALID_ARG
    assert L.tkv_decode_reduce(C.byref(d), fake, 4, 2, 64, fake, fake, C.c_size_t(16), null) == tkv.TKV_ERR_WORKSPACE_TOO_SMALL
    assert L.tkv_decode_reduce(C.byref(d), fake, 4, 0, 64, fake, fake, big, null) == tkv.TKV_OK


def test_gather_dequant_validates_before_launch():
    L = tkv.lib()
    d = tkv.tkv_desc.make(8, 4, 4)
    buf = (C.c_uint8 * 4096)()
    base = (C.addressof(buf) + 255) & ~255
    p = C.c_void_p(base)
    def call(**kw):
        a = dict(pool=p, bm=p, wp=p, wd=p, n_work=C.c_int32(1), Ko=p, Vo=p, n_tokens=C.c_int32(64), st=None, stream=None)
        a.update(kw)
        return L.tkv_gather_dequant(C.byref(d), a["pool"], a["bm"], a["wp"], a["wd"], a["n_work"], a["Ko"], a["Vo"],
                                    a["n_tokens"], a["st"], a["stream"])
    assert call(n_work=C.c_int32(0)) == tkv.TKV_OK                       # nothing to do: no launch
    assert call(n_work=C.c_int32(-1)) == tkv.TKV_ERR_INVALID_ARG
    assert call(n_tokens=C.c_int32(-1)) == tkv.TKV_ERR_INVALID_ARG
    assert call(pool=None) == tkv.TKV_ERR_INVALID_ARG
    assert call(Ko=None) == tkv.TKV_ERR_INVALID_ARG
    assert call(wd=None) == tkv.TKV_ERR_INVALID_ARG
    assert call(Ko=C.c_void_p(base + 8)) == tkv.TKV_ERR_INVALID_ARG       # output rows must be 16-byte aligned
    assert call(pool=C.c_void_p(base + 16)) == tkv.TKV_ERR_INVALID_ARG    # pool must be 256-byte aligned
    bad = tkv.tkv_desc.make(8, 4, 4)
    bad.head_dim = 64
    assert L.tkv_gather_dequant(C.byref(bad), p, p, p, p, 0, p, p, 0, None, None) != tkv.TKV_OK


def test_residual_routing_matches_the_oracle_and_keeps_blocks_whole(oracle):
    """Residual policy of per-channel INT2 keys (Sec. 3.2.1): the library's rewrite against the oracle's."""
    rng = np.random.default_rng(31)
    for _ in range(200):
        n = int(rng.integers(0, 400))
        b = rng.choice([2, 4], n, p=[0.7, 0.3]).astype(np.uint8)
        got = tkv.tkv_route_residual(b)
        assert np.array_equal(got, oracle.route_residual(b))
        assert int((got == 2).sum()) % 32 == 0
    assert tkv.tkv_route_residual(np.uint8([2] * 31)).tolist() == [4] * 31
    with pytest.raises(tkv.TkvError) as e:
        tkv.tkv_route_residual(np.uint8([2, 3]))
    assert e.value.status == tkv.TKV_ERR_BAD_BITS
    # in place
    b = np.uint8([2] * 40)
    p = C.c_void_p(b.ctypes.data)
    assert tkv.lib().tkv_route_residual(p, 40, p) == tkv.TKV_OK and b.tolist() == [2] * 32 + [4] * 8


def test_per_channel_key_mode_is_validated():
    d = tkv.tkv_desc.make(2, 4, 4, int2_key_axis=tkv.TKV_KEYS_PER_CHANNEL)
    assert tkv.tkv_pool_bytes(d) == tkv.tkv_pool_bytes(tkv.tkv_desc.make(2, 4, 4))      # same record size
    bad = tkv.tkv_desc.make(2, 4, 4, int2_key_axis=2)
    assert tkv.tkv_pool_bytes(bad) == 0
    h = C.c_void_p()
    assert tkv.lib().tkv_alloc_create(C.byref(bad), 0, C.byref(h)) == tkv.TKV_ERR_BAD_SHAPE
    a, s = tkv.tkv_alloc_create(d, 0), tkv.tkv_seq_create()
    with pytest.raises(tkv.TkvError) as e:
        tkv.tkv_plan_append(a, s, np.uint8([2] * 33))            # INT2 tokens must come in blocks of 32
    assert e.value.status == tkv.TKV_ERR_INVALID_ARG
    assert tkv.tkv_seq_n_tokens(s, 2) == 0 and tkv.tkv_alloc_free_count(a, 2) == 4
    slots, wp, ws = tkv.tkv_plan_append(a, s, tkv.tkv_route_residual(np.uint8([2] * 33)))
    assert tkv.tkv_seq_n_tokens(s, 2) == 32 and tkv.tkv_seq_n_tokens(s, 4) == 1
    # decode plan: an INT2 token count that is not a multiple of 32 cannot come from this mode
    ip = np.int32([0, 1])
    with pytest.raises(tkv.TkvError):
        tkv.tkv_plan_decode(d, ip, np.int32([33]), np.int32([0]), 1)
    items, sip = tkv.tkv_plan_decode(d, ip, np.int32([32]), np.int32([0]), 1)
    assert items.tolist() == [[0, 0, 1, 0]]
    tkv.tkv_seq_destroy(s)
    tkv.tkv_alloc_destroy(a)


def test_record_and_mix_probes_validate_before_launch():
    L = tkv.lib()
    d = tkv.tkv_desc.make(8, 4, 4)
    fake, null = C.c_void_p(0x1000), C.c_void_p(None)
    rec = lambda **kw: L.tkv_probe_decode_reads(C.byref(kw.get("desc", d)), kw.get("pool", fake), fake, fake, fake, fake,
                                                kw.get("items", fake), kw.get("n_items", 4), kw.get("batch", 2), kw.get("walk", 1),
                                                null, null)
    assert rec(n_items=0) == tkv.TKV_OK
    assert rec(desc=tkv.tkv_desc.make(8, 0, 0)) == tkv.TKV_OK                      # an empty pool: nothing to read
    assert rec(desc=tkv.tkv_desc.make(8, 4, 4, head_dim=64)) == tkv.TKV_ERR_BAD_SHAPE
    assert rec(n_items=-1) == tkv.TKV_ERR_INVALID_ARG
    assert rec(walk=2) == tkv.TKV_ERR_INVALID_ARG
    assert rec(pool=null) == tkv.TKV_ERR_INVALID_ARG
    assert rec(pool=C.c_void_p(0x1010)) == tkv.TKV_ERR_INVALID_ARG
    assert rec(items=null) == tkv.TKV_ERR_INVALID_ARG                            # walk = 1 reads the items
    assert rec(batch=0) == tkv.TKV_ERR_INVALID_ARG
    mix = lambda src=fake, dst=fake, n=64, r=4, w=1: L.tkv_probe_stream_mix(src, dst, n, r, w, null)
    assert mix(n=0) == tkv.TKV_OK
    assert mix(r=3) == tkv.TKV_ERR_INVALID_ARG and mix(r=1, w=2) == tkv.TKV_ERR_INVALID_ARG
    assert mix(n=24) == tkv.TKV_ERR_INVALID_ARG
    assert mix(src=null) == tkv.TKV_ERR_INVALID_ARG and mix(dst=C.c_void_p(0x1008)) == tkv.TKV_ERR_INVALID_ARG


def test_stream_read_probe_validates_before_launch():
    L = tkv.lib()
    assert L.tkv_probe_stream_read(None, 0, None, None) == tkv.TKV_OK                 # nothing to read
    assert L.tkv_probe_stream_read(None, 64, None, None) == tkv.TKV_ERR_INVALID_ARG
    assert L.tkv_probe_stream_read(C.c_void_p(0x1008), 64, None, None) == tkv.TKV_ERR_INVALID_ARG   # misaligned
    assert L.tkv_probe_stream_read(C.c_void_p(0x1000), 24, None, None) == tkv.TKV_ERR_INVALID_ARG   # not a multiple of 16
