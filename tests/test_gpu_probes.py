"""The measurement probes of the library run on the GPU without touching what they read, and tkv_probe_stream_mix
writes what its declaration says (a fold of what it read)."""
import numpy as np
import pytest
import torch

from paper_2605_17170_amd import harness, tkv

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    from tests import gpu_common
    return gpu_common


def test_record_probe_reads_the_plan_and_leaves_the_pool_alone(G):
    q, K, V, seq_bits = G.random_case(41, [700, 0, 130, 64], 8, 2)
    cache, _ = G.check_append(seq_bits, K, V, 2)
    try:
        before = cache.pool.clone()
        cache.plan_decode(9)
        d_items = cache._plan[0]
        for walk in (True, False):
            tkv.tkv_probe_decode_reads(cache.desc, cache.pool, cache.d_page_indptr, cache.d_page_ids, cache.d_n_tok2,
                                       cache.d_n_tok4, d_items, 4, walk)
        # without the page walk the tables are not needed
        L = tkv.lib()
        import ctypes as C
        st = L.tkv_probe_decode_reads(C.byref(cache.desc), C.c_void_p(cache.pool.data_ptr()), None, None, None, None, None,
                                      int(d_items.shape[0]), 4, 0, None, None)
        assert st == tkv.TKV_OK
        torch.cuda.synchronize()
        assert torch.equal(before, cache.pool)
    finally:
        cache.close()


@pytest.mark.parametrize("unit", [16, 4096 + 16, 1 << 20])
def test_stream_mix_writes_the_fold_of_what_it_read(G, unit):
    g = torch.Generator(device=G.DEV)
    g.manual_seed(unit)
    src = torch.randint(0, 256, (4 * unit,), dtype=torch.uint8, device=G.DEV, generator=g)
    dst = torch.zeros(4 * unit + 64, dtype=torch.uint8, device=G.DEV)
    dst[4 * unit:] = 0x5A
    tkv.tkv_probe_stream_mix(src, dst, unit, 1, 1)
    torch.cuda.synchronize()
    assert torch.equal(dst[:unit], src[:unit]) and bool((dst[unit:4 * unit] == 0).all())
    tkv.tkv_probe_stream_mix(src, dst, unit, 4, 1)
    torch.cuda.synchronize()
    want = src[:unit] ^ src[unit:2 * unit] ^ src[2 * unit:3 * unit] ^ src[3 * unit:]
    assert torch.equal(dst[:unit], want) and bool((dst[unit:4 * unit] == 0).all())
    tkv.tkv_probe_stream_mix(src, dst, unit, 1, 4)
    torch.cuda.synchronize()
    for k in range(4):
        assert torch.equal(dst[k * unit:(k + 1) * unit], src[:unit])
    assert bool((dst[4 * unit:] == 0x5A).all()), "bytes behind the destination were written"
