"""The decode phase of a request (Sec. 3.2.3, "Decode", phase 2): after the prefill has been cached, every
step writes the keys and values of one newly generated token per sequence at INT4 into the sequence's open
INT4 page (a new page when the open one is full: the page table grows by one entry) and then attends over the
whole cache.  Checked here through the C ABI, step by step, against the oracle: every pool byte after the
last step, and the attention output at chosen steps, with per-token and with per-channel INT2 keys."""
import numpy as np
import pytest
import torch

from paper_2605_17170_amd import harness, tkv
from paper_2605_17170_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import gpu_common
    return gpu_common


@pytest.mark.parametrize("axis", [tkv.TKV_KEYS_PER_TOKEN, tkv.TKV_KEYS_PER_CHANNEL])
def test_generation_loop_grows_the_int4_stream(G, axis):
    from oracle import tkv_oracle as orc
    H, Hq, B, steps = 2, 8, 3, 70
    prefill = [150, 61, 0]                      # the third sequence starts empty
    total = [n + steps for n in prefill]
    q_all, K, V, seq_bits = G.random_case(21, total, Hq, H, f4=0.3)
    # token rows: sequence b owns rows [row0[b], row0[b] + total[b]); its first prefill[b] rows are the prompt
    row0 = np.concatenate([[0], np.cumsum(total)])[:-1]
    tags = [np.concatenate([seq_bits[b][:prefill[b]], np.full(steps, 4, np.uint8)]) for b in range(B)]   # generated tokens are INT4
    desc = tkv.tkv_desc.make(H, 16, 16, int2_key_axis=axis)
    a = tkv.tkv_alloc_create(desc, 5)
    seqs = [tkv.tkv_seq_create() for _ in range(B)]
    dev = G.DEV
    pool = torch.full((tkv.tkv_pool_bytes(desc),), 0xA5, dtype=torch.uint8, device=dev)
    bmap = torch.zeros(32, dtype=torch.uint8, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    dK, dV = harness.bf16_tensor(K, dev), harness.bf16_tensor(V, dev)
    bits = np.zeros(K.shape[0], np.uint8)       # the widths the tokens are stored at, filled in as they arrive
    slots = np.full(K.shape[0], -1, np.int64)
    blocks = []

    def append(b, lo, hi):
        """Rows [lo, hi) of sequence b arrive as one chunk."""
        t = tags[b][lo:hi]
        if axis == tkv.TKV_KEYS_PER_CHANNEL:
            t = tkv.tkv_route_residual(t)
            assert np.array_equal(t, orc.route_residual(tags[b][lo:hi]))
            blocks.append(orc.int2_blocks(t, row0[b] + lo))
        base = int(row0[b] + lo)
        bits[base:base + hi - lo] = t
        sl, wp, ws = tkv.tkv_plan_append(a, seqs[b], t, token_base=base)
        slots[base:base + hi - lo] = sl
        if wp.size:
            tkv.tkv_quantize_append(desc, pool, bmap, dK, dV, torch.from_numpy(bits).to(dev),
                                    torch.from_numpy(wp).to(dev), torch.from_numpy(ws).to(dev), status)

    def decode(n_gen):
        ids = [tkv.tkv_seq_page_ids(s) for s in seqs]
        indptr = np.concatenate([[0], np.cumsum([i.size for i in ids])]).astype(np.int32)
        n2 = np.array([tkv.tkv_seq_n_tokens(s, 2) for s in seqs], np.int32)
        n4 = np.array([tkv.tkv_seq_n_tokens(s, 4) for s in seqs], np.int32)
        items, sip = tkv.tkv_plan_decode(desc, indptr, n2, n4, 5)
        t = lambda x: torch.from_numpy(np.ascontiguousarray(x)).to(dev)
        out = torch.empty((B, Hq, 128), dtype=torch.float32, device=dev)
        ws = torch.empty(max(16, tkv.tkv_decode_workspace_bytes(desc, items.shape[0], Hq)), dtype=torch.uint8, device=dev)
        tkv.tkv_decode_attention(desc, pool, bmap, harness.bf16_tensor(q_all, dev), t(indptr), t(np.concatenate(ids).astype(np.int32)),
                                 t(n2), t(n4), t(items), t(sip), G.SM, out, ws, status)
        torch.cuda.synchronize()
        assert int(status.item()) == 0
        # oracle: the tokens cached so far, in row order per sequence
        rows = np.concatenate([np.arange(row0[b], row0[b] + prefill[b] + n_gen) for b in range(B)])
        Kh, Vh = dequantised()
        lens = [prefill[b] + n_gen for b in range(B)]
        ip = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        ref = orc.attention_f64(wl.bf16_bits_to_f32(q_all).astype(np.float64), np.ascontiguousarray(Kh[rows]),
                                np.ascontiguousarray(Vh[rows]), ip, G.SM)
        G.assert_close(out.cpu().numpy(), ref, "after %d generated tokens" % n_gen)

    def quantised():
        b = np.where(bits == 0, 4, bits).astype(np.uint8)        # rows that have not arrived yet: any width
        Kq, Vq = orc.quantize(K, b), orc.quantize(V, b)
        tok = np.concatenate(blocks) if blocks else np.zeros((0, 32), np.int64)
        bs = bz = None
        if axis == tkv.TKV_KEYS_PER_CHANNEL:
            bs, bz = orc.quantize_k_channel(K, tok, Kq[0])
            Kq[1][bits == 2] = 0
            Kq[2][bits == 2] = 0
        return Kq, Vq, tok, bs, bz

    def dequantised():
        Kq, Vq, tok, bs, bz = quantised()
        Kh = orc.dequantize(*Kq)
        if bs is not None:
            orc.dequantize_k_channel(Kq[0], tok, bs, bz, Kh)
        return Kh, orc.dequantize(*Vq)

    for b in range(B):
        append(b, 0, prefill[b])
    decode(0)
    for step in range(steps):
        for b in range(B):
            append(b, prefill[b] + step, prefill[b] + step + 1)
        if step + 1 in (1, 2, 3, 64, 65, steps):
            decode(step + 1)
    # every byte of the pool after the last step
    Kq, Vq, tok, bs, bz = quantised()
    o_pool = np.full(pool.numel(), 0xA5, np.uint8)
    o_map = np.zeros(32, np.uint8)
    orc.pack_pool(o_pool, o_map, H, 16, 16, slots, bits, Kq, Vq)
    if bs is not None:
        orc.put_kblocks(o_pool, H, 16, slots, tok, bs, bz)
    assert np.array_equal(bmap.cpu().numpy(), o_map)
    g_pool = pool.cpu().numpy()
    assert np.array_equal(g_pool, o_pool), "pool bytes differ at %s" % np.nonzero(g_pool != o_pool)[0][:8].tolist()
    # the INT4 stream grew by whole pages as the open page filled
    for b in range(B):
        n4 = tkv.tkv_seq_n_tokens(seqs[b], 4)
        assert n4 == int((bits[row0[b]:row0[b] + total[b]] == 4).sum()) and tkv.tkv_seq_n_pages(seqs[b], 4) == -(-n4 // 64)
    for s in seqs:
        tkv.tkv_seq_destroy(s)
    tkv.tkv_alloc_destroy(a)
