#!/usr/bin/env python3
"""Benchmark of the TriAxialKV decode / append hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config cfg5] [--legs all|none] [--no-cpu]

Prints ONE JSON line.  The headline workload is cfg5, the largest single-GPU
configuration of the baseline file: a Llama-3-70B-shaped decode step, 80
layers, 64 query heads on 8 kv heads, batch 32, context lengths lognormal
between 4K and 128K tokens, tokens at INT2 or INT4 by their tag (2.6 bits on
average).  A "step" is the decode attention of ONE generated token through
all 80 layers: 80 x tkv_decode_attention (split-K kernel + cross-split
reduction, through the C ABI) back to back on one stream, each layer reading
its own paged pool (page table shared by the layers, K/V of every layer drawn
from its own seed).  The pools (64 GB) are built before the timed region by
tkv_quantize_append and are resident in HBM; a layer's pool (805 MB) is far
larger than the 256 MB Infinity Cache, so every step reads from HBM.

value = effective KV bytes per second = (96 B per INT2 token + 160 B per INT4
token) x kv heads, summed over the batch and the layers, divided by the step
time.  The other configurations of the baseline file run as legs of the same
line (one layer each, pools rotated over copies larger than the Infinity
Cache): cfg2, cfg3 and cfg1 decode steps, the cfg4 append.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published
METRIC = "effective KV GB/s + µs/decode step (mixed INT2/INT4), % of HBM peak"
SHAPES = {
    "cfg1": "cfg1 (B=1, Hq=4, Hkv=1, d=128, ctx 2048, 1 layer)",
    "cfg2": "cfg2 (Qwen3-VL-32B-shaped layer: B=8, Hq=64, Hkv=8, d=128, ctx 32768, 1 layer)",
    "cfg3": "cfg3 (B=4, Hq=4, Hkv=1, d=128, ctx 102400, 1 layer, pool sized for 16 sequences)",
    "cfg5": "cfg5 (Llama-3-70B-shaped decode step: 80 layers, B=32, Hq=64, Hkv=8, d=128, ctx lognormal 4K..128K)",
}


def csrc_hash() -> str:
    """Hash of the kernel sources: ties a profile summary to the binary it was taken from."""
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2605_17170_amd", "csrc")
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".cpp", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(d, name), "rb").read())
    return h.hexdigest()[:12]


def read_traffic(name):
    """HBM bytes per launch of the dominant kernel from a committed rocprofv3 --pmc summary (profiles/<name>),
    or None when there is none or it was taken from other kernel sources than the ones in the tree."""
    path = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(path):
        return None
    val, sha = None, None
    for line in open(path):
        if line.startswith("hbm_bytes_per_launch"):
            val = float(line.split("=")[1])
        if line.startswith("csrc_sha"):
            sha = line.split("=")[1].strip()
    return val if sha == csrc_hash() else None


def timed(fn, steps, warmup, min_warm_s=0.030):
    """Runs fn(i) at least `warmup` times untimed, then `steps` times; returns (ms per step from one pair of HIP events on the launch stream
    around the `steps` timed calls, as an array of one element; wall ms per step between two synchronisations).
    Nothing is recorded between the steps: an event per step costs 3-10 us of stream time each, which a step of
    tens of microseconds would carry as if it were its own."""
    import torch
    # untimed: `warmup` calls, and more of them until the device has been busy for min_warm_s (a short warm-up
    # leaves the clocks low: the first 12 ms of cfg2 steps after 1 ms of warm-up run 20 % slower than the next 12 ms)
    t_warm = time.perf_counter()
    n_warm = 0
    while n_warm < warmup or (time.perf_counter() - t_warm < min_warm_s and n_warm < 100000):
        fn(n_warm)
        n_warm += 1
        if n_warm % 64 == 0:
            torch.cuda.synchronize()
    torch.cuda.synchronize()
    first, last = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    first.record()
    for i in range(steps):
        fn(i)
    last.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / steps
    return np.array([first.elapsed_time(last) / steps]), wall


def frac(nbytes, ms):
    return nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS


def cpu_baseline(w, q_host, K_host, V_host, nseq, note):
    """The oracle's decode attention, as it stands, on the host cores, on the leading `nseq` sequences."""
    from oracle import tkv_oracle as orc
    bits = w.all_bits()
    ip = w.seq_indptr
    T = int(ip[nseq])
    Kq = orc.quantize(K_host[:T], bits[:T])
    Vq = orc.quantize(V_host[:T], bits[:T])
    sm = float(np.float32(1.0 / math.sqrt(128.0)))
    t0 = time.perf_counter()
    orc.attention_quantized(q_host[:nseq], Kq, Vq, ip[:nseq + 1], sm)
    dt = time.perf_counter() - t0
    nbytes = w.n_kv_heads * (96 * int((bits[:T] == 2).sum()) + 160 * int((bits[:T] == 4).sum()))
    return {"value": nbytes / dt / 1e9, "unit": "GB/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": "%s: %d of %d sequences (%d tokens, all heads), decode attention only, %.2f s" % (note, nseq, w.batch, T, dt),
            "seconds": dt, "bytes": nbytes}


def decode_leg(name, steps, warmup, key_axis=0, n_layers=1):
    """Decode step of one configuration on device-generated K/V.  n_layers > 1: one pool per layer, a step walks all
    layers; otherwise the pool is rotated over copies whose total exceeds 768 MB (cold protocol)."""
    import torch
    from paper_2605_17170_amd import harness, tkv
    from paper_2605_17170_amd import workloads as wl
    dev = torch.device("cuda:0")
    w = wl.config(name)
    pool_factor = 4.0 if name == "cfg3" else 1.0
    cache = harness.PagedCache(w.n_kv_heads, w.bits, dev, pool_factor=pool_factor, shuffle_seed=w.seed + 1, key_axis=key_axis,
                               alloc_pool=False)
    target = harness.default_target_items(w.n_kv_heads, dev)
    t0 = time.perf_counter()
    items, _ = cache.plan_decode(target)
    plan_us = (time.perf_counter() - t0) * 1e6
    kv_bytes = cache.kv_bytes()
    pools, qs = [], []
    app_ms = []
    for layer in range(n_layers):
        K, V = harness.device_kv(w.n_tokens, w.n_kv_heads, w.seed * 1000 + layer, dev)
        pool = torch.empty(cache.pool_bytes, dtype=torch.uint8, device=dev)
        if layer == 0:
            per, _ = timed(lambda i: cache.append(K, V, pool=pool), 3, 1)
            app_ms = float(np.median(per))
        else:
            cache.append(K, V, pool=pool)
        pools.append(pool)
        qs.append(harness.device_q(w.batch, w.n_q_heads, w.seed * 1000 + layer, dev))
        del K, V
    if n_layers == 1:
        n_copies = max(1, min(8, int(math.ceil(768e6 / max(cache.pool_bytes, 1)))))
        pools += [pools[0].clone() for _ in range(n_copies - 1)]
        qs = qs * n_copies
    else:
        # one plain device copy of known size (a pool): the calibration point of the rocprofv3 byte counters
        calib = pools[0].clone()
        del calib
    torch.cuda.synchronize()
    assert int(cache.status.item()) == 0
    out = torch.empty((w.batch, w.n_q_heads, 128), dtype=torch.float32, device=dev)
    ws = cache.workspace(w.n_q_heads)
    n_pools = len(pools)

    # the calls with their arguments marshalled once: the timed loops then cost one C call per launch
    steps_c = [cache.decode(qs[k], out=out, workspace=ws, pool=pools[k], prepare=True) for k in range(n_pools)]
    splits_c = [cache.decode_split(qs[k], workspace=ws, pool=pools[k], prepare=True) for k in range(n_pools)]
    if n_layers > 1:
        def step(i):
            for call in steps_c:
                call()

        def split_only(i):
            for call in splits_c:
                call()
    else:
        def step(i):
            steps_c[i % n_pools]()

        def split_only(i):
            splits_c[i % n_pools]()

    # the headline (80 layers a step) warms up by exactly `warmup` steps; the single-layer legs by at least 30 ms
    min_warm = 0.0 if n_layers > 1 else 0.030
    per, wall_ms = timed(step, steps, warmup, min_warm)
    sp, sp_wall = timed(split_only, steps, warmup, min_warm)
    assert int(cache.status.item()) == 0
    launches = n_layers
    res = {
        "workload": SHAPES[name], "n_layers": n_layers, "batch": w.batch, "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads,
        "tokens": w.n_tokens, "int4_token_share": float((cache.tag_bits == 4).mean()),
        "kv_bytes_per_layer": kv_bytes, "kv_bytes_per_step": kv_bytes * n_layers,
        "work_items": int(items.shape[0]), "work_items_target": int(target), "pools": n_pools,
        "ms_per_step": wall_ms, "us_per_layer": wall_ms * 1e3 / n_layers,
        "GBps": kv_bytes * n_layers / (wall_ms * 1e-3) / 1e9, "frac_of_hbm_peak": frac(kv_bytes * n_layers, wall_ms),
        "kernel_us": float(np.mean(sp)) * 1e3 / launches, "kernel_frac_of_hbm_peak": frac(kv_bytes * n_layers, float(np.mean(sp))),
        "plan_decode_host_us": plan_us,
        "append_whole_context_ms": app_ms,
    }
    return res, (w, cache, pools, qs, out, ws)


def append_leg(name, steps=5, warmup=2):
    """tkv_quantize_append (and the prefill gather back) of a whole workload: tokens/s and read + written GB/s."""
    import torch
    from paper_2605_17170_amd import harness
    from paper_2605_17170_amd import workloads as wl
    dev = torch.device("cuda:0")
    w = wl.config(name)
    cache = harness.PagedCache(w.n_kv_heads, w.bits, dev, pool_factor=2.0 if name == "cfg4" else 1.0, shuffle_seed=w.seed + 1)
    K, V = harness.device_kv(w.n_tokens, w.n_kv_heads, w.seed * 1000, dev)
    per, _ = timed(lambda i: cache.append(K, V), steps, warmup)
    ms = float(np.median(per))
    rd, wr = 2 * K.numel() * 2, cache.kv_bytes()
    gK = torch.empty((w.n_tokens, w.n_kv_heads, 128), dtype=torch.float16, device=dev)
    gV = torch.empty_like(gK)
    gper, _ = timed(lambda i: cache.gather(gK, gV), steps, warmup)
    gms = float(np.median(gper))
    assert int(cache.status.item()) == 0
    # ceilings for these byte mixes: plain streams that read 4 bytes per byte written (append) and the reverse (gather)
    from paper_2605_17170_amd import tkv
    unit = (wr // 16) * 16
    src = K.view(torch.uint8).reshape(-1)
    big = torch.empty(4 * unit, dtype=torch.uint8, device=dev)
    mix41 = tkv.tkv_probe_stream_mix(big, cache.pool, unit, 4, 1, prepare=True)
    mix14 = tkv.tkv_probe_stream_mix(cache.pool, big, unit, 1, 4, prepare=True)
    m41 = float(np.median(timed(lambda i: mix41(), steps, warmup)[0]))
    m14 = float(np.median(timed(lambda i: mix14(), steps, warmup)[0]))
    del big, src
    res = {"workload": "%s: %d new bf16 K and V tokens, %d kv heads, INT4 token share %.2f, randomly allocated pages"
                       % (name, w.n_tokens, w.n_kv_heads, w.f4()),
           "append_ms": ms, "tokens_per_s": w.n_tokens / (ms * 1e-3), "GBps_read_plus_write": (rd + wr) / (ms * 1e-3) / 1e9,
           "frac_of_hbm_peak": frac(rd + wr, ms), "bytes_read": rd, "bytes_written": wr,
           "prefill_gather_ms": gms, "prefill_gather_GBps_read_plus_write": (wr + 2 * gK.numel() * 2) / (gms * 1e-3) / 1e9,
           "prefill_gather_frac_of_hbm_peak": frac(wr + 2 * gK.numel() * 2, gms),
           "stream_read4_write1_GBps": 5 * unit / (m41 * 1e-3) / 1e9, "stream_read1_write4_GBps": 5 * unit / (m14 * 1e-3) / 1e9,
           "ceiling_note": "tkv_probe_stream_mix: plain 128-bit streams (ordinary loads, non-temporal stores) of the same size in the byte ratio of the append "
                           "(reads 4, writes 1) and of the gather (reads 1, writes 4); the second one overwrites the pool, "
                           "after the measurements that needed it"}
    cache.close()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed steps (default: 20 for cfg5, 200 otherwise)")
    ap.add_argument("--warmup", type=int, default=0, help="warm-up steps (default: 3 for cfg5, 20 otherwise)")
    ap.add_argument("--config", default="cfg5", choices=["cfg1", "cfg2", "cfg3", "cfg5"], help="headline workload")
    ap.add_argument("--legs", default="all", choices=["all", "none"])
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_17170_amd import harness, tkv

    tkv.lib()   # fail loudly if the HIP library is missing
    torch.cuda.set_device(0)
    head = args.config
    steps = args.steps or (20 if head == "cfg5" else 200)
    warmup = args.warmup or (3 if head == "cfg5" else 20)
    n_layers = 80 if head == "cfg5" else 1
    main_res, (w, cache, pools, qs, out, ws) = decode_leg(head, steps, warmup, n_layers=n_layers)

    # speed-of-light probe: a plain 128-bit (non-temporal) streaming read of the same pools, same order
    probe, _ = timed(lambda i: tkv.tkv_probe_stream_read(pools[i % len(pools)]), 40, 5)
    stream_read = cache.pool_bytes / (float(np.mean(probe)) * 1e-3) / 1e9
    kv_layer, kv_step = main_res["kv_bytes_per_layer"], main_res["kv_bytes_per_step"]
    kernel_us = main_res["kernel_us"]
    # the decode kernel's own reads without its arithmetic: records fetched one per wavefront at a time, first with
    # computed addresses (what the memory system gives this access pattern), then through the item and page tables as
    # the kernel does (its memory skeleton, start-up chain and ragged end included)
    d_items = cache._plan[0]
    rec_calls = {walk: [tkv.tkv_probe_decode_reads(cache.desc, p_, cache.d_page_indptr, cache.d_page_ids, cache.d_n_tok2,
                                                   cache.d_n_tok4, d_items, w.batch, walk, prepare=True) for p_ in pools]
                 for walk in (False, True)}
    rec_t = {walk: float(np.mean(timed(lambda i: rec_calls[walk][i % len(pools)](), 40, 5)[0])) for walk in (False, True)}
    record_read = cache.pool_bytes / (rec_t[False] * 1e-3) / 1e9
    skeleton = kv_layer / (rec_t[True] * 1e-3) / 1e9
    res = {
        "metric": METRIC, "value": main_res["GBps"], "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": main_res["ms_per_step"], "us_per_decode_step": main_res["ms_per_step"] * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u2/u4 codes, f16 MFMA operands, f32 accumulate", "data": "synthetic",
        "config": {k: main_res[k] for k in ("workload", "n_layers", "batch", "n_q_heads", "n_kv_heads", "tokens", "int4_token_share",
                                            "kv_bytes_per_layer", "kv_bytes_per_step", "work_items", "work_items_target", "pools")},
        "pct_of_hbm_peak": 100.0 * main_res["frac_of_hbm_peak"],
        "us_per_layer": main_res["us_per_layer"],
        "plan_decode": {"host_us": main_res["plan_decode_host_us"],
                        "note": "tkv_plan_decode on the host, once: the plan stays valid until a sequence gains a page (every 64 decoded "
                                "tokens per sequence at most) and is shared by the 80 layers, so it costs host_us / (64 x 80) per layer step"},
        "roofline": {"bound": "hbm", "achieved": kv_layer / (kernel_us * 1e-6) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": kv_layer / (kernel_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                     "traffic": read_traffic("decode_%s_hbm_traffic.txt" % head),
                     "kernel": "tkv_decode_kernel", "kernel_us": kernel_us, "bytes_per_launch": kv_layer,
                     "stream_read_GBps": stream_read, "frac_of_stream_read": kv_layer / (kernel_us * 1e-6) / 1e9 / stream_read,
                     "record_read_GBps": record_read, "memory_skeleton_GBps": skeleton, "memory_skeleton_us": rec_t[True] * 1e3,
                     "csrc_sha": csrc_hash(),
                     "note": "tkv_decode_kernel launched by itself (tkv_decode_split) over the same pools in the same order, mean "
                             "interval per launch from HIP events around the timed launches on the launch stream; algorithmic bytes "
                             "per launch = 96 B/INT2 token + 160 B/INT4 token per kv head of one layer; traffic = HBM bytes per launch "
                             "from rocprofv3 FETCH_SIZE + WRITE_SIZE (profiles/), null unless that summary was taken from these kernel "
                             "sources; stream_read_GBps = a plain 128-bit streaming read of the same pools with non-temporal loads, as the kernel uses (tkv_probe_stream_read); "
                             "record_read_GBps = the pool's records read whole, one per wavefront at a time, addresses computed; "
                             "memory_skeleton = the same reads through the items and page tables, i.e. the decode kernel without "
                             "its arithmetic (tkv_probe_decode_reads, walk = 0 / 1)"},
    }
    if not args.no_cpu:
        # the oracle on a bounded sample: the leading sequences of layer 0 (device-generated K/V copied to the host)
        budget_tok = max(1, 8_000_000 // w.n_kv_heads)   # a whole layer of cfg5 (877 779 tokens on 8 kv heads)
        ip = w.seq_indptr
        nseq = 1
        while nseq < w.batch and ip[nseq + 1] <= budget_tok:
            nseq += 1
        T = int(ip[nseq])
        K, V = harness.device_kv(w.n_tokens, w.n_kv_heads, w.seed * 1000, torch.device("cuda:0"))
        Kh = K[:T].view(torch.int16).cpu().numpy().view(np.uint16)
        Vh = V[:T].view(torch.int16).cpu().numpy().view(np.uint16)
        qh = qs[0][:nseq].view(torch.int16).cpu().numpy().view(np.uint16)
        del K, V
        cb = cpu_baseline(w, qh, Kh, Vh, nseq, "layer 0 of %s" % head)
        if n_layers > 1:
            cb["extrapolated_seconds_per_step"] = cb["seconds"] * kv_step / cb["bytes"]
            cb["sample"] += "; extrapolated to the whole step (all sequences, %d layers) by bytes" % n_layers
        res["cpu_baseline"] = cb
    del pools, qs
    cache.close()
    torch.cuda.empty_cache()

    if args.legs == "all":
        legs = {}
        for name in ("cfg2", "cfg3", "cfg1"):
            if name == head:
                continue
            r, keep = decode_leg(name, 200, 20)
            keep[1].close()
            del keep
            torch.cuda.empty_cache()
            legs[name + "_decode"] = r
        r, keep = decode_leg("cfg2", 200, 20, key_axis=tkv.TKV_KEYS_PER_CHANNEL)
        keep[1].close()
        del keep
        torch.cuda.empty_cache()
        r["workload"] += ", INT2 keys quantised per channel over 32-token blocks (tkv_desc.int2_key_axis)"
        legs["cfg2_decode_per_channel_int2_keys"] = r
        legs["cfg4_append"] = append_leg("cfg4")
        legs["cfg2_append"] = append_leg("cfg2")
        # decode-phase append: one generated token per sequence written at INT4 into the open page
        import torch as _t
        dev = _t.device("cuda:0")
        B, H = 32, 8
        small = harness.PagedCache(H, [np.full(100, 4, np.uint8)] * B, dev, pool_factor=2.0)
        t0 = time.perf_counter()
        plans = [tkv.tkv_plan_append(small.alloc, s, np.uint8([4]), b) for b, s in enumerate(small.seqs)]
        plan1_us = (time.perf_counter() - t0) * 1e6
        wp1 = _t.from_numpy(np.concatenate([p[1] for p in plans])).to(dev)
        ws1 = _t.from_numpy(np.concatenate([p[2] for p in plans])).to(dev)
        b1 = _t.full((B,), 4, dtype=_t.uint8, device=dev)
        K1, V1 = harness.device_kv(B, H, 5, dev)
        app1 = tkv.tkv_quantize_append(small.desc, small.pool, small.bit_map, K1, V1, b1, wp1, ws1, small.status, prepare=True)
        one, _ = timed(lambda i: app1(), 200, 20)
        assert int(small.status.item()) == 0
        legs["decode_phase_append"] = {"us_per_step": float(np.median(one)) * 1e3, "plan_host_us": plan1_us,
                                       "note": "tkv_quantize_append of one new INT4 token per sequence (%d sequences, %d kv heads): interval "
                                               "between back-to-back launches of the prepared call (one C call each; bounded below by the "
                                               "host's launch rate; the kernel's own duration is in the rocprofv3 kernel trace)" % (B, H)}
        small.close()
        res["legs"] = legs
    print(json.dumps(res))


if __name__ == "__main__":
    main()
