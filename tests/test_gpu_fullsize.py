"""Parity at the full sizes of the benchmark configurations, in the launch
configuration bench.py times (default work-item count): every pool byte
against the oracle-packed pool, and every decode output against the oracle's
fp64 attention.  cfg5 (80 layers) is checked on its first, middle and last
layer at full shape; the layers differ only by their seed."""
import time

import numpy as np
import pytest

from paper_2605_17170_amd import harness
from paper_2605_17170_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import gpu_common
    return gpu_common


def _full(G, name, layer=0, pool_factor=1.0):
    from oracle import tkv_oracle as orc
    t0 = time.time()
    w = wl.config(name)
    q, K, V, _ = w.make_inputs(layer)
    t1 = time.time()
    cache = harness.PagedCache(w.n_kv_heads, w.bits, G.DEV, pool_factor=pool_factor, shuffle_seed=w.seed + 1, fill=0xA5)
    try:
        g_pool, g_map = G.gpu_append(cache, K, V)
        out = G.gpu_decode(cache, q, harness.default_target_items(w.n_kv_heads))
        t2 = time.time()
        bits = cache.tag_bits
        Kq, Vq = orc.quantize(K, bits), orc.quantize(V, bits)
        o_pool, o_map = G.oracle_pool(cache, Kq, Vq, 0xA5)
        assert np.array_equal(g_map, o_map)
        assert np.array_equal(g_pool, o_pool), "pool bytes differ at %s" % np.nonzero(g_pool != o_pool)[0][:8].tolist()
        t3 = time.time()
        ref = G.decode_ref(q, Kq, Vq, w.seq_lens)
        t4 = time.time()
        ratio = G.assert_close(out, ref, name)
        print("  %s: %d tokens, gen %.1fs gpu %.1fs oracle quantize+pack %.1fs attention %.1fs" %
              (name, w.n_tokens, t1 - t0, t2 - t1, t3 - t2, t4 - t3), flush=True)
        return ratio
    finally:
        cache.close()


def test_cfg2_full(G):
    _full(G, "cfg2")


def test_cfg3_full_scattered_pool(G):
    _full(G, "cfg3", pool_factor=4.0)      # pool sized for 16 sequences, 4 in use, pages scattered


@pytest.mark.parametrize("layer", [0, 39, 79])
def test_cfg5_layer_full(G, layer):
    _full(G, "cfg5", layer=layer)
