#!/usr/bin/env python3
"""Benchmark of the TriAxialKV decode / append hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config cfg2]

Prints ONE JSON line.  A "step" is one decode-attention step of one layer over
the whole batch of the workload: split-K decode kernel + cross-split reduction
(tkv_decode_attention through the C ABI), reading a paged INT2/INT4 cache that
tkv_quantize_append built from the workload's bf16 K/V before the timed
region (that append is timed too and reported under "append").  Inputs are
resident in HBM when timing starts.  To keep the 256 MB Infinity Cache from
serving the pool, the steps rotate over several identical copies of the pool
whose total size exceeds 512 MB ("cold" protocol); a warm number (one copy)
is reported beside it.

value = effective KV bytes per second = (96 B per INT2 token + 160 B per INT4
token) x kv heads, summed over the batch, divided by the step time.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published


def _events(n):
    import torch
    return [torch.cuda.Event(enable_timing=True) for _ in range(n)]


def time_steps(fn, steps, warmup):
    """Per-step GPU durations (ms) from HIP events on the launch stream, and
    the wall time of the whole timed region bracketed by synchronize()."""
    import torch
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    ev = _events(steps + 1)
    t0 = time.perf_counter()
    ev[0].record()
    for i in range(steps):
        fn(i)
        ev[i + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    per = np.array([ev[i].elapsed_time(ev[i + 1]) for i in range(steps)])
    return per, wall


def cpu_baseline(w, q, K, V, max_seconds=30.0):
    """The oracle's decode attention, timed as it stands on the host cores, on
    a bounded sample of the same workload (whole sequences, all heads)."""
    from oracle import tkv_oracle as orc
    bits = w.all_bits()
    ip = w.seq_indptr
    # sample: as many leading sequences as ~4M tokens x kv heads allow (a few seconds of scalar work)
    budget_tok = max(1, 4_000_000 // w.n_kv_heads)
    nseq = 1
    while nseq < w.batch and ip[nseq + 1] <= budget_tok:
        nseq += 1
    T = int(ip[nseq])
    Kq = orc.quantize(K[:T], bits[:T])
    Vq = orc.quantize(V[:T], bits[:T])
    sm = float(np.float32(1.0 / math.sqrt(128.0)))
    t0 = time.perf_counter()
    orc.attention_quantized(q[:nseq], Kq, Vq, ip[:nseq + 1], sm)
    dt = time.perf_counter() - t0
    nbytes = w.n_kv_heads * (96 * int((bits[:T] == 2).sum()) + 160 * int((bits[:T] == 4).sum()))
    return {"value": nbytes / dt / 1e9, "unit": "GB/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": "%d of %d sequences (%d tokens, all heads), decode attention only, %.2f s" % (nseq, w.batch, T, dt)}


def read_traffic(name):
    """HBM bytes per launch of the dominant kernel from committed rocprofv3
    --pmc summaries (profiles/<name>), or None."""
    path = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(path):
        return None
    for line in open(path):
        if line.startswith("hbm_bytes_per_launch"):
            return float(line.split("=")[1])
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="cfg2", choices=["cfg1", "cfg2", "cfg3", "cfg5"])
    ap.add_argument("--scale", type=float, default=1.0, help="shrink context lengths (debug only; makes the line invalid)")
    ap.add_argument("--target-items", type=int, default=0)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_17170_amd import harness, tkv
    from paper_2605_17170_amd import workloads as wl

    tkv.lib()   # fail loudly if the HIP library is missing
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = wl.config(args.config, args.scale)
    q, K, V, _ = w.make_inputs()
    pool_factor = 4.0 if args.config == "cfg3" else 1.0
    cache = harness.PagedCache(w.n_kv_heads, w.bits, dev, pool_factor=pool_factor, shuffle_seed=w.seed + 1)
    dK, dV, dq = harness.bf16_tensor(K, dev), harness.bf16_tensor(V, dev), harness.bf16_tensor(q, dev)

    # ---- append leg (builds the cache the decode steps read)
    app_per, _ = time_steps(lambda i: cache.append(dK, dV), 5, 2)
    app_ms = float(np.median(app_per))
    app_read = 2 * K.size * 2
    app_write = cache.kv_bytes()
    assert int(cache.status.item()) == 0

    # ---- prefill gather leg (dequantises the whole cached context back into fp16 rows)
    gK = torch.empty((w.n_tokens, w.n_kv_heads, 128), dtype=torch.float16, device=dev)
    gV = torch.empty_like(gK)
    gat_per, _ = time_steps(lambda i: cache.gather(gK, gV), 5, 2)
    gat_ms = float(np.median(gat_per))
    gat_bytes = cache.kv_bytes() + 2 * gK.numel() * 2
    assert int(cache.status.item()) == 0
    del gK, gV

    # ---- decode leg
    target = args.target_items or harness.default_target_items(w.n_kv_heads, dev)
    t0 = time.perf_counter()
    items, _ = cache.plan_decode(target)
    plan_us = (time.perf_counter() - t0) * 1e6
    kv_bytes = cache.kv_bytes()
    pool_bytes = cache.pool.numel()
    n_copies = max(1, min(8, int(math.ceil(768e6 / max(pool_bytes, 1)))))
    pools = [cache.pool] + [cache.pool.clone() for _ in range(n_copies - 1)]
    out = torch.empty((w.batch, w.n_q_heads, 128), dtype=torch.float32, device=dev)
    ws = cache.workspace(w.n_q_heads)

    def step_cold(i):
        cache.decode(dq, out=out, workspace=ws, pool=pools[i % n_copies])

    def step_warm(i):
        cache.decode(dq, out=out, workspace=ws, pool=pools[0])

    def split_cold(i):
        cache.decode_split(dq, workspace=ws, pool=pools[i % n_copies])

    per, wall = time_steps(step_cold, args.steps, args.warmup)
    ms_per_step = wall * 1e3 / args.steps
    # the dominant kernel by itself (tkv_decode_kernel = the split launch), same rotation, HIP events per launch
    split_per, _ = time_steps(split_cold, args.steps, args.warmup)
    ev_ms = float(np.mean(split_per))
    warm_per, _ = time_steps(step_warm, min(args.steps, 50), 5)
    # speed-of-light probe: a plain 128-bit streaming read of the same pool copies, same rotation
    probe_per, _ = time_steps(lambda i: tkv.tkv_probe_stream_read(pools[i % n_copies]), 40, 5)
    stream_read = pool_bytes / (float(np.mean(probe_per)) * 1e-3) / 1e9
    assert int(cache.status.item()) == 0
    value = kv_bytes / (ms_per_step * 1e-3) / 1e9

    res = {
        "metric": "effective KV GB/s + \u00b5s/decode step (mixed INT2/INT4), % of HBM peak",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "us_per_decode_step": ms_per_step * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u2/u4 codes, f16 MFMA operands, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": args.config + (" (Qwen3-VL-32B-shaped layer: B=8, Hq=64, Hkv=8, d=128, ctx 32768)"
                                              if args.config == "cfg2" else ""),
                   "batch": w.batch, "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads,
                   "tokens": w.n_tokens, "int4_token_share": w.f4(), "kv_bytes_per_step": kv_bytes,
                   "work_items": int(items.shape[0]), "pool_copies_rotated": n_copies, "scale": args.scale},
        "pct_of_hbm_peak": 100.0 * value / HBM_PEAK_GBS,
        "warm_cache": {"us_per_step": float(np.median(warm_per)) * 1e3,
                       "GBps": kv_bytes / (float(np.median(warm_per)) * 1e-3) / 1e9,
                       "note": "single pool copy; may be served by the 256 MB Infinity Cache"},
        "plan_decode_host_us": plan_us,
        "append": {"ms": app_ms, "tokens_per_s": w.n_tokens / (app_ms * 1e-3),
                   "GBps_read_plus_write": (app_read + app_write) / (app_ms * 1e-3) / 1e9,
                   "pct_of_hbm_peak": 100.0 * (app_read + app_write) / (app_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                   "note": "tkv_quantize_append of the whole context (bf16 K,V read + packed pages written), outside the timed steps"},
        "prefill_gather": {"ms": gat_ms, "tokens_per_s": w.n_tokens / (gat_ms * 1e-3),
                           "GBps_read_plus_write": gat_bytes / (gat_ms * 1e-3) / 1e9,
                           "pct_of_hbm_peak": 100.0 * gat_bytes / (gat_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                           "note": "tkv_gather_dequant of the whole context (packed pages read + fp16 K,V rows written), outside the timed steps"},
        "roofline": {"bound": "hbm", "achieved": kv_bytes / (ev_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": kv_bytes / (ev_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "traffic": read_traffic("decode_%s_hbm_traffic.txt" % args.config),
                     "kernel": "tkv_decode_kernel", "kernel_us": ev_ms * 1e3,
                     "stream_read_GBps": stream_read, "frac_of_stream_read": kv_bytes / (ev_ms * 1e-3) / 1e9 / stream_read,
                     "note": "tkv_decode_kernel launched by itself (tkv_decode_split), mean of HIP-event intervals "
                             "between back-to-back launches; algorithmic bytes = 96 B/INT2 token + 160 B/INT4 token "
                             "per kv head; traffic = HBM bytes per launch from rocprofv3 FETCH_SIZE + WRITE_SIZE; "
                             "stream_read_GBps = a plain 128-bit streaming read of the same pool copies (tkv_probe_stream_read), "
                             "what the memory system delivers to a read-only scan on this box"},
    }
    # ---- the same workload with the paper's own INT2 key scheme (keys per channel over 32-token blocks,
    #      tokens that do not fill a block stored at INT4): append, gather and decode legs
    del pools
    cache.close()
    kc = harness.PagedCache(w.n_kv_heads, w.bits, dev, pool_factor=pool_factor, shuffle_seed=w.seed + 1,
                            key_axis=tkv.TKV_KEYS_PER_CHANNEL)
    kc_app, _ = time_steps(lambda i: kc.append(dK, dV), 5, 2)
    gK = torch.empty((w.n_tokens, w.n_kv_heads, 128), dtype=torch.float16, device=dev)
    gV = torch.empty_like(gK)
    kc_gat, _ = time_steps(lambda i: kc.gather(gK, gV), 5, 2)
    del gK, gV
    kc.plan_decode(target)
    kc_pools = [kc.pool] + [kc.pool.clone() for _ in range(n_copies - 1)]
    kc_ws = kc.workspace(w.n_q_heads)
    _, kc_wall = time_steps(lambda i: kc.decode(dq, out=out, workspace=kc_ws, pool=kc_pools[i % n_copies]),
                            args.steps, args.warmup)
    kc_split, _ = time_steps(lambda i: kc.decode_split(dq, workspace=kc_ws, pool=kc_pools[i % n_copies]),
                             args.steps, args.warmup)
    assert int(kc.status.item()) == 0
    kc_bytes = kc.kv_bytes()
    kc_ms = kc_wall * 1e3 / args.steps
    res["per_channel_int2_keys"] = {
        "us_per_decode_step": kc_ms * 1e3, "GBps": kc_bytes / (kc_ms * 1e-3) / 1e9,
        "pct_of_hbm_peak": 100.0 * kc_bytes / (kc_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "kernel_us": float(np.mean(kc_split)) * 1e3,
        "kernel_frac_of_hbm_peak": kc_bytes / (float(np.mean(kc_split)) * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "kv_bytes_per_step": kc_bytes, "int4_token_share": float((kc.tag_bits == 4).mean()),
        "append_ms": float(np.median(kc_app)), "prefill_gather_ms": float(np.median(kc_gat)),
        "note": "same workload, tkv_desc.int2_key_axis = per channel; same cold-pool protocol"}
    # ---- decode-phase append: one generated token per sequence written at INT4 into the open page
    small = harness.PagedCache(w.n_kv_heads, [np.full(100, 4, np.uint8)] * w.batch, dev, pool_factor=2.0)
    t0 = time.perf_counter()
    plans = [tkv.tkv_plan_append(small.alloc, s, np.uint8([4]), b) for b, s in enumerate(small.seqs)]
    plan1_us = (time.perf_counter() - t0) * 1e6
    wp1 = torch.from_numpy(np.concatenate([p[1] for p in plans])).to(dev)
    ws1 = torch.from_numpy(np.concatenate([p[2] for p in plans])).to(dev)
    b1 = torch.full((w.batch,), 4, dtype=torch.uint8, device=dev)
    one_per, _ = time_steps(lambda i: tkv.tkv_quantize_append(small.desc, small.pool, small.bit_map, dK[:w.batch], dV[:w.batch],
                                                              b1, wp1, ws1, small.status), 50, 5)
    assert int(small.status.item()) == 0
    res["decode_phase_append"] = {"us_per_step": float(np.median(one_per)) * 1e3, "plan_host_us": plan1_us,
                                  "note": "tkv_quantize_append of one new INT4 token per sequence (%d sequences, %d kv heads), "
                                          "interval between back-to-back launches through the Python binding (bounded below by the host's call "
                                          "overhead; the kernel's own duration is in the rocprofv3 kernel trace); host planning of the %d "
                                          "single-token appends beside it"
                                          % (w.batch, w.n_kv_heads, w.batch)}
    small.close()
    if not args.no_cpu:
        res["cpu_baseline"] = cpu_baseline(w, q, K, V)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
