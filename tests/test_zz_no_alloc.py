"""tkv_decode_attention_static (the entry point for callers that cannot allocate: partials in a fixed device
array inside the library) against tkv_decode_attention on the same inputs, through the C ABI: two calls in a
row, the second with a smaller input, so that what the first call left in the shared array must not leak
into the second; then the size limit."""
import numpy as np
import pytest
import torch

from paper_2605_17170_amd import harness, tkv

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import gpu_common
    return gpu_common


def _both(G, seed, seq_lens, hq, hkv, target):
    q, K, V, seq_bits = G.random_case(seed, seq_lens, hq, hkv)
    cache, (Kq, Vq) = G.check_append(seq_bits, K, V, hkv)
    try:
        ref = G.decode_ref(q, Kq, Vq, seq_lens)
        cache.plan_decode(target)
        dq = harness.bf16_tensor(q, G.DEV)
        want = cache.decode(dq)
        got = torch.full_like(want, float("nan"))
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        cache.decode_static(dq, got)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert int(cache.status.item()) == 0
        got, want = got.cpu().numpy(), want.cpu().numpy()
        G.assert_close(got, ref, "static entry vs oracle, %s" % (seq_lens,))
        G.assert_close(want, ref, "workspace entry vs oracle, %s" % (seq_lens,))
        # the two entry points launch the same kernels on the same plan
        assert np.allclose(got, want, rtol=1e-2, atol=2e-3)
        print("  max |static - workspace| = %.3e" % float(np.abs(got - want).max()), flush=True)
    finally:
        cache.close()


def test_static_entry_matches_workspace_entry_twice_second_call_smaller(G):
    _both(G, 61, [5000, 900, 0, 2500], 32, 4, 96)    # 96 items x 32 heads: 1.6 MB of partials
    _both(G, 62, [700, 130], 8, 2, 5)                # far fewer, shorter items: most of the array keeps the first call's data


def test_static_entry_rejects_more_partials_than_its_array_holds(G):
    q, K, V, seq_bits = G.random_case(63, [64 * 600], 64, 8)
    cache = harness.PagedCache(8, seq_bits, G.DEV)
    try:
        cache.plan_decode(600)      # 600 items x 64 heads x 520 B = 20 MB > 16 MiB
        n_items = cache._plan[2].shape[0]
        assert tkv.tkv_decode_workspace_bytes(cache.desc, n_items, 64) > tkv.TKV_DECODE_STATIC_SCRATCH_BYTES
        out = torch.zeros((1, 64, 128), dtype=torch.float32, device=G.DEV)
        with pytest.raises(tkv.TkvError) as e:
            cache.decode_static(harness.bf16_tensor(q, G.DEV), out)
        assert e.value.status == tkv.TKV_ERR_WORKSPACE_TOO_SMALL
        torch.cuda.synchronize()
        assert float(out.abs().max()) == 0.0      # nothing was launched
    finally:
        cache.close()
