#!/usr/bin/env python3
"""Decode-step benchmark: fused score -> top-k -> sparse decode on one MI355X.

One "step" is one pass of the whole hot path (absb_decode_fused: estimation over the INT4
centroid codes, per-head Top-K, split-K attention over the selected blocks, LSE merge) over one
batch of synthetic input that is already resident in HBM.  The default workload is the headline
one: batch 1, 128K context, Llama-3.1-8B-shaped layer (32 query / 8 KV heads, d = 128, fp16),
per-head block sizes from {8,...,128}, budget 4096 tokens.

Cold-cache discipline: the step cycles over R independent layer instances (own KV pages, codes,
query) so that no step re-reads lines the previous ones left in L2 / Infinity Cache.

Prints ONE JSON line.  `value` = useful (algorithmic) bytes per step / step time, in GB/s.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published peak
METRIC = "decode attention µs/step/layer + achieved HBM GB/s at 128K ctx (8B-shaped GQA)"
# HBM bytes moved by one absb_sparse_decode call on the headline workload, from rocprofv3 --pmc
# (FETCH_SIZE, then WRITE_SIZE, each scaled by a 1 GiB copy in the same run): partials kernel
# 17.06 MB read + 1.06 MB written, merge kernel 1.19 MB + 0.01 MB.
# Source: profiles/decode_fused_config3_hbm_counters.md
HEADLINE_TRAFFIC_BYTES = 19_320_000


def useful_bytes(wl, plan_off, sel_cnt):
    """Algorithmic bytes of one step: what the method itself must move.
    score : INT4 codes of every centroid (d/2 bytes each) + per-channel scales + queries
    select: the index list
    decode: K and V rows of the selected tokens + page-table entries touched + queries + outputs
    Intermediate arrays (int32 scores, split-K partials) are not counted."""
    d, e = wl.head_dim, 2
    nseg = wl.batch * wl.num_kv_heads
    total = int(plan_off[-1])
    b_score = total * (d // 2) + nseg * d * 4 + wl.batch * wl.num_q_heads * d * e
    b_select = int(sel_cnt.sum()) * 4
    tokens = 0
    pt_entries = 0
    for s in range(nseg):
        b, h = divmod(s, wl.num_kv_heads)
        B = int(wl.block_size[h])
        k = int(sel_cnt[s])
        tokens += min(k * B, int(wl.seq_lens[b]))
        pt_entries += k * max(1, B // wl.page_size)
    b_kv = tokens * 2 * d * e
    b_decode = b_kv + pt_entries * 4 + 2 * wl.batch * wl.num_q_heads * d * e
    return dict(score=b_score, select=b_select, decode=b_decode, kv=b_kv, total=b_score + b_select + b_decode)


def time_loop(fn, n_warm, n_steps):
    """Average milliseconds per call of fn(i), timed with events on the launch stream."""
    import torch
    for i in range(n_warm):
        fn(i)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for i in range(n_steps):
        fn(i)
    ev1.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / n_steps
    return ev0.elapsed_time(ev1) / n_steps, wall


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--config", type=int, default=3, help="workload recipe 1..5 (3 = headline)")
    ap.add_argument("--rotate", type=int, default=0, help="layer instances cycled through (0 = auto: >= 2 GiB of KV)")
    ap.add_argument("--context", type=int, default=None)
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--budget", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--stages", action="store_true", help="also time each entry point on its own")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="run one device-to-device copy of this many MiB first (a kernel of known traffic, for "
                         "scaling hardware byte counters collected with rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_12110_amd import absb, synth
    from paper_2605_12110_amd.device import DeviceWorkload
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    absb.load()
    torch.cuda.set_device(0)

    if args.copy_calibration > 0:
        src = torch.full((args.copy_calibration << 20,), 7, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    base_seed = {1: 0, 2: 1, 3: 2, 4: 3, 5: 4}[args.config]
    wl0 = synth.make_workload(args.config, context=args.context, batch=args.batch, budget=args.budget)
    R = args.rotate
    if R <= 0:
        R = max(1, min(8, -(-(2 << 30) // wl0.kv_bytes())))
    insts = [DeviceWorkload(wl0)]
    for r in range(1, R):
        wl = synth.make_workload(args.config, context=args.context, batch=args.batch, budget=args.budget,
                                 seed=base_seed + 100 * r)
        insts.append(DeviceWorkload(wl))
        if r > 0:
            insts[-1].wl.k_cache = insts[-1].wl.v_cache = None     # free host copies of the extra instances
    for dw in insts:
        dw.build()
    torch.cuda.synchronize()

    # one untimed step per instance to learn the selection sizes (for the byte count)
    ub = []
    for dw in insts:
        dw.decode_fused()
        torch.cuda.synchronize()
        ub.append(useful_bytes(dw.wl, dw.plan.cent_off, dw.sel_cnt.cpu().numpy()))
    mean_bytes = {k: float(np.mean([u[k] for u in ub])) for k in ub[0]}

    def step(i):
        insts[i % R].decode_fused(want_sel=False)

    ms, wall_ms = time_loop(step, args.warmup, args.steps)
    us = ms * 1e3
    gbps = mean_bytes["total"] / (ms * 1e-3) / 1e9

    # dominant stage on its own: sparse decode (split-K partials + merge) on the fused step's selection
    def step_decode(i):
        insts[i % R].sparse_decode()

    ms_dec, _ = time_loop(step_decode, args.warmup, args.steps)
    dec_gbps = mean_bytes["decode"] / (ms_dec * 1e-3) / 1e9
    stages = {"sparse_decode_us": ms_dec * 1e3}
    if args.stages:
        ms_sc, _ = time_loop(lambda i: insts[i % R].score(), args.warmup, args.steps)
        ms_tk, _ = time_loop(lambda i: insts[i % R].topk(), args.warmup, args.steps)
        stages.update(score_us=ms_sc * 1e3, topk_us=ms_tk * 1e3)

    wl = wl0
    headline = args.config == 3 and args.context is None and args.batch is None and args.budget is None
    result = {
        "metric": METRIC,
        "value": round(gbps, 2),
        "unit": "GB/s",
        "us_per_step": round(us, 3),
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms, 6),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16" if wl.dtype == synth.F16 else "bf16",
        "data": "synthetic",
        "config": {
            "workload": f"config{args.config}: batch {wl.batch}, context {int(wl.seq_lens.max())}, "
                        f"{wl.num_q_heads}q/{wl.num_kv_heads}kv heads, d={wl.head_dim}, page {wl.page_size}, "
                        f"block sizes {wl.block_size.tolist()}, budget {int(wl.budget.max())} tokens",
            "entry_point": "absb_decode_fused",
            "layer_instances_rotated": R,
            "resident_kv_bytes": int(sum(i.k_cache.numel() * 2 * 2 for i in insts)),
            "useful_bytes_per_step": {k: int(v) for k, v in mean_bytes.items()},
            "fraction_of_hbm_peak": round(gbps / HBM_PEAK_GBPS, 4),
            "host_wall_us_per_step": round(wall_ms * 1e3, 2),
            "stages": {k: round(v, 3) for k, v in stages.items()},
        },
        "roofline": {
            "bound": "hbm",
            # the event-timed unit is the entry point absb_sparse_decode = the dominant kernel
            # (decode_partial_kernel, which reads the K/V rows) plus the small LSE merge kernel
            "kernel": "decode_partial_kernel + decode_merge_kernel (one absb_sparse_decode call)",
            "achieved": round(dec_gbps, 2),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(dec_gbps / HBM_PEAK_GBPS, 4),
            "algorithmic_bytes_per_launch": int(mean_bytes["decode"]),
            "us_per_launch": round(ms_dec * 1e3, 3),
            "traffic": HEADLINE_TRAFFIC_BYTES if headline else None,
        },
    }

    if not args.no_cpu_baseline:
        from oracle import oracle as O
        st = O.build_centroids(wl0)
        O.decode_step(wl0, st)                       # warm
        t0 = time.perf_counter()
        n = 0
        while True:
            O.decode_step(wl0, st)
            n += 1
            el = time.perf_counter() - t0
            if el > 10.0 or n >= 2000:
                break
        cpu_s = el / n
        result["cpu_baseline"] = {
            "value": round(ub[0]["total"] / cpu_s / 1e9, 3),
            "unit": "GB/s",
            "us_per_step": round(cpu_s * 1e6, 1),
            "cores": O.num_threads(),
            "kind": "oracle",
            "sample": f"{n} full steps (score -> top-k -> attention over the selection) of the same workload, "
                      f"instance 0, prebuilt codes, {el:.1f} s of wall time",
        }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
