#!/usr/bin/env python3
"""Decode-step benchmark: fused score -> top-k -> sparse decode on one MI355X.

One "step" is one pass of the whole hot path (absb_decode_fused: estimation over the INT4
centroid codes, per-head Top-K, split-K attention over the selected blocks, LSE merge) over one
batch of synthetic input that is already resident in HBM.  The default workload is the headline
one: batch 1, 128K context, Llama-3.1-8B-shaped layer (32 query / 8 KV heads, d = 128, fp16),
per-head block sizes from {8,...,128}, budget 4096 tokens.

Cold-cache discipline: the step cycles over R resident copies of the layer (own KV pages, codes,
query, workspace: same contents at other addresses), with R sized by the bytes a step TOUCHES:
R x useful bytes >= 2 x the 256 MB last-level cache, so that no step finds lines that an earlier
visit of the same copy left in L2 or in the Infinity Cache.  All copies hold the same data, so one
block-size table, one selection and one byte count describe every step; copy 0 is checked against
the oracle after the timed loop and every other copy against copy 0.

Timing: the K timed steps are captured into a HIP graph (kernels only) and replayed between two
events on the launch stream, so the figure is the GPU's step time, not the Python loop's call
rate; the eager loop is timed too and reported next to it.

Default run: prints ONE JSON line.  `value` = useful (algorithmic) bytes per step / step time, GB/s.
`--matrix`: runs every benchmark configuration (and the config-5 budget sweep with selection
recall and error against dense attention) and prints a markdown table instead.
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
LAST_LEVEL_CACHE_BYTES = 256 << 20   # Infinity Cache; the L2s (8 x 4 MB) are smaller
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "decode_fused_config3_hbm_counters.md")
BASE_SEED = {1: 0, 2: 1, 3: 2, 4: 3, 5: 4}


def kernel_sources_sha16():
    """Hash of the library's sources: ties a counter measurement under profiles/ to the kernels it was taken on."""
    import hashlib
    h = hashlib.sha256()
    src = os.path.join(ROOT, "paper_2605_12110_amd", "csrc")
    for name in sorted(os.listdir(src)):
        h.update(open(os.path.join(src, name), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(kernel):
    """HBM bytes per launch of `kernel` on the headline workload as rocprofv3 --pmc counted them
    (FETCH_SIZE + WRITE_SIZE, scaled by a copy of known size), from the committed profile summary,
    or None when that summary was taken on other kernel sources than the ones in this tree."""
    import re
    try:
        text = open(TRAFFIC_PROFILE).read()
    except OSError:
        return None
    m = re.search(r"traffic_bytes_per_launch\[" + re.escape(kernel) + r"\]\s*=\s*(\d+)\s+kernel_sources_sha16\s*=\s*([0-9a-f]{16})", text)
    if not m or m.group(2) != kernel_sources_sha16():
        return None
    return int(m.group(1))


def useful_bytes(wl, plan_off, sel_cnt, vectors=1, per_query_head=False):
    """Algorithmic bytes of one step: what the method itself must move.
    score : INT4 codes of every block (d/2 bytes per vector: one for mean pooling, two for
            max-min pooling) + per-channel scales + queries
    select: the index list
    decode: K and V rows of the selected tokens + page-table entries touched + queries + outputs
    Intermediate arrays (int32 scores, split-K partials) are not counted.
    With per-query-head selection every query head scans its KV head's codes and reads the rows of
    its own list: the method itself then moves G times the codes and up to G times the rows."""
    d, e = wl.head_dim, 2
    rk = wl.group if per_query_head else 1              # selection segments per KV head
    hsel = wl.num_kv_heads * rk
    nseg = wl.batch * hsel
    total = int(plan_off[-1])
    b_score = vectors * rk * (total * (d // 2) + wl.batch * wl.num_kv_heads * d * 4) + wl.batch * wl.num_q_heads * d * e
    b_select = int(sel_cnt.sum()) * 4
    tokens = 0
    pt_entries = 0
    for s in range(nseg):
        b, hs = divmod(s, hsel)
        h = hs // rk
        B = int(wl.block_size[h])
        k = int(sel_cnt[s])
        tokens += min(k * B, int(wl.seq_lens[b]))
        pt_entries += k * max(1, B // wl.page_size)
    b_kv = tokens * 2 * d * e
    b_decode = b_kv + pt_entries * 4 + 2 * wl.batch * wl.num_q_heads * d * e
    return dict(score=b_score, select=b_select, decode=b_decode, kv=b_kv, total=b_score + b_select + b_decode)


def time_loop(fn, n_warm, n_steps):
    """Average milliseconds per call of fn(i) in an eager loop, timed with events on the launch stream;
    also the host's wall time per call."""
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


def time_graph(fn, period, n_warm, n_steps):
    """Average milliseconds per call of fn(i), i = 0 .. n_steps-1 (fn only depends on i % period), with
    the calls captured into HIP graphs and replayed between two events on the launch stream: exactly
    n_steps calls are timed, as floor(n_steps / period) replays of a graph of `period` calls plus one
    graph holding the remainder.  The calls enqueue kernels only (no memset, allocation or
    synchronisation), which is what a captured graph may hold."""
    import torch
    for i in range(n_warm):
        fn(i)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()

    def capture(count, first):
        g = torch.cuda.CUDAGraph()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                for i in range(count):
                    fn(first + i)
        torch.cuda.current_stream().wait_stream(side)
        return g
    full, rem = divmod(n_steps, period)
    g_full = capture(period, 0) if full else None
    g_rem = capture(rem, full * period) if rem else None
    for g in (g_full, g_rem):                     # first replay uploads the graph: not timed
        if g is not None:
            g.replay()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(full):
        g_full.replay()
    if g_rem is not None:
        g_rem.replay()
    ev1.record()
    torch.cuda.synchronize()
    return ev0.elapsed_time(ev1) / n_steps


def per_step_percentiles(fn, n_steps):
    """Per-step durations from an event between consecutive eager steps: (p10, median, p90) in us
    (each includes the event's own cost, about 2-3 us)."""
    import torch
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(n_steps + 1)]
    torch.cuda.synchronize()
    evs[0].record()
    for i in range(n_steps):
        fn(i)
        evs[i + 1].record()
    torch.cuda.synchronize()
    d = np.array([evs[i].elapsed_time(evs[i + 1]) * 1e3 for i in range(n_steps)])
    return float(np.percentile(d, 10)), float(np.median(d)), float(np.percentile(d, 90))


def make_instances(config, *, context=None, batch=None, budget=None, rotate=0, uniform_block=None, max_bytes=64 << 30,
                   block_repr=0, selection=0, opts=None, block_sizes=None, **synth_kw):
    """R resident copies of one workload (the same data at R places in HBM), the centroid store built
    once and copied.  R (`rotate`, 0 = auto) is sized by what a step touches: R x useful bytes of a
    step >= 2 x the last-level cache, at most 256 copies and `max_bytes` of device memory."""
    import torch
    from paper_2605_12110_amd import synth
    from paper_2605_12110_amd.device import DeviceWorkload
    kw = dict(context=context, batch=batch, budget=budget, uniform_block=uniform_block)
    if block_sizes is not None:
        kw["block_sizes"] = block_sizes
    kw.update(synth_kw)
    wl0 = synth.make_workload(config, **kw)
    first = DeviceWorkload(wl0, block_repr=block_repr, selection=selection, opts=opts)
    first.build()
    first.decode_fused()
    torch.cuda.synchronize()
    ub = useful_bytes(wl0, first.plan.cent_off, first.sel_cnt.cpu().numpy(), block_repr + 1, selection == 1)
    R = rotate
    if R <= 0:
        R = -(-2 * LAST_LEVEL_CACHE_BYTES // max(ub["total"], 1)) + 1
    per_copy = 2 * first.k_cache.numel() * 2 + first.workspace.numel() + first.codes.numel()
    R = max(1, min(R, 256, max_bytes // max(per_copy, 1)))
    insts = [first] + [first.clone() for _ in range(R - 1)]
    torch.cuda.synchronize()
    return wl0, insts, ub


def measure(wl0, insts, ub, steps, warmup, stages=True, percentiles=False):
    """Times the fused step (graph replay and eager) and, with `stages`, every entry point on its own."""
    import torch
    from paper_2605_12110_amd import absb
    R = len(insts)

    def step(i):
        insts[i % R].decode_fused(want_sel=False)

    ms = time_graph(step, R, warmup, steps)
    ms_eager, wall_ms = time_loop(step, min(warmup, 10), steps)
    form = absb.absb_step_form_used(insts[0].layer, insts[0].batch)
    out = dict(ms=ms, ms_eager=ms_eager, wall_ms=wall_ms, bytes=ub, R=R, form=form,
               launches=3 if form == absb.STEP_PER_STAGE else 1)
    # every instance has completed a fused step on its workspace, so its split counters are zero and
    # absb_sparse_decode with that promise is exactly one launch of the attention kernel, on the
    # fused step's own selection
    for dw in insts:
        dw.decode_fused()
        dw.batch.opts.counters_zero = 1
    torch.cuda.synchronize()
    try:
        st = {"sparse_decode_us": time_graph(lambda i: insts[i % R].sparse_decode(), R, warmup, steps) * 1e3}
    finally:
        for dw in insts:
            dw.batch.opts.counters_zero = 0
    if stages:
        st["score_us"] = time_graph(lambda i: insts[i % R].score(), R, warmup, steps) * 1e3
        st["topk_us"] = time_graph(lambda i: insts[i % R].topk(), R, warmup, steps) * 1e3
    out["ms_decode"] = st["sparse_decode_us"] * 1e-3
    out["stages"] = st
    if percentiles:
        out["p10_med_p90_us"] = per_step_percentiles(step, min(steps, 200))
    return out


def stream_read_ceiling(gib=2, reps=10):
    """GB/s of a plain 128-bit-load read of `gib` GiB (larger than every cache), event-timed."""
    import torch
    from paper_2605_12110_amd import absb
    buf = torch.full((gib << 30,), 3, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    ms, _ = time_loop(lambda i: absb.absb_stream_read(buf, sink), 2, reps)
    del buf
    torch.cuda.empty_cache()
    return (gib << 30) / (ms * 1e-3) / 1e9


def _time_oracle(fn, seconds, max_n=2000):
    t0 = time.perf_counter()
    n = 0
    while True:
        fn()
        n += 1
        el = time.perf_counter() - t0
        if el > seconds or n >= max_n:
            return el / n, n, el


def verify_against_oracle(insts, ref):
    """One more step of every resident copy: copy 0 against the oracle's step on the same inputs
    (selection bit for bit, output within tolerance), every other copy against copy 0 (same inputs,
    so the same bits).  The number above is only worth reporting if the timed path computes the right
    thing, on every copy it was timed on."""
    import torch
    for dw in insts:
        dw.sel_idx.fill_(-7)
        dw.out.fill_(float("nan"))
        dw.decode_fused()
    torch.cuda.synchronize()
    dw = insts[0]
    K = dw.sel_stride
    sel_ok = bool(np.array_equal(dw.sel_cnt.cpu().numpy(), ref["sel_cnt"]) and
                  np.array_equal(dw.sel_idx.cpu().numpy(), ref["sel_idx"][:, :K]))
    err = float(np.abs(dw.out_f32().astype(np.float64) - ref["out"]).max())
    tol = 2e-3 if dw.wl.dtype == 0 else 1e-2
    status = max(d.status() for d in insts)
    same = all(torch.equal(d.sel_idx, dw.sel_idx) and torch.equal(d.sel_cnt, dw.sel_cnt) and torch.equal(d.out, dw.out)
               for d in insts[1:])
    if not (sel_ok and err <= tol and status == 0 and same):
        raise SystemExit(f"bench.py: the timed path disagrees with the oracle (selection bit-exact: {sel_ok}, "
                         f"max |out - oracle| = {err:.3e}, tolerance {tol:.0e}, status word {status}, "
                         f"all {len(insts)} copies agree: {same})")
    return {"selection_bit_exact": sel_ok, "max_abs_err_out": float(f"{err:.3e}"), "tolerance": tol,
            "copies_checked": len(insts),
            "what": "one fused step of every resident copy after the timed loops: copy 0 against the oracle's step, "
                    "the others bit for bit against copy 0"}


def cpu_baseline(wl0, bytes0, seconds=10.0, block_repr=0, check=None, selection=0):
    from oracle import oracle as O
    t0 = time.perf_counter()
    st = O.build_centroids(wl0, block_repr)
    build_s = time.perf_counter() - t0
    ref = O.decode_step(wl0, st, group_max=selection == 2)        # warm
    verified = None
    if check is not None:
        if selection == 1:     # every query head its own group: the oracle runs the method on that model
            view = O.per_query_head_view(wl0)
            ref = O.decode_step(view, O.build_centroids(view, block_repr))
        verified = verify_against_oracle(check, ref)
    cpu_s, n, el = _time_oracle(lambda: O.decode_step(wl0, st), seconds)
    threads = O.num_threads()
    O.set_threads(1)
    try:
        one_s, n1, el1 = _time_oracle(lambda: O.decode_step(wl0, st), min(3.0, seconds))
    finally:
        O.set_threads(threads)
    return {
        "value": round(bytes0["total"] / cpu_s / 1e9, 3),
        "unit": "GB/s",
        "us_per_step": round(cpu_s * 1e6, 1),
        "cores": threads,
        "kind": "oracle",
        "sample": f"{n} full steps (score -> top-k -> attention over the selection) of the same workload, "
                  f"instance 0, prebuilt codes, {el:.1f} s of wall time",
        "single_thread_us_per_step": round(one_s * 1e6, 1),
        "single_thread_sample": f"{n1} steps, {el1:.1f} s",
        "oracle_build_seconds_once": round(build_s, 3),
        "verified": verified,
    }


def synth_workload(cfg):
    from paper_2605_12110_amd import synth
    return synth.make_workload(cfg)


def run_matrix(args):
    """Every benchmark configuration, then the config-5 sweep (uniform 16 vs adaptive block sizes)."""
    import torch
    from oracle import oracle as O
    rows = []
    print("| workload | batch | dtype | launches/step | useful MB/step | us/step (mean; p10/med/p90) | GB/s | % of 8 TB/s | "
          "decode stage us | decode GB/s | oracle us/step (cores) |")
    print("|---|---|---|---|---|---|---|---|---|---|---|", flush=True)
    for cfg in (1, 2, 3, 4):
        wl0, insts, ub = make_instances(cfg)
        m = measure(wl0, insts, ub, args.steps, args.warmup, stages=False, percentiles=True)
        cb = cpu_baseline(wl0, m["bytes"], seconds=3.0)
        gb = m["bytes"]["total"] / (m["ms"] * 1e-3) / 1e9
        dgb = m["bytes"]["decode"] / (m["ms_decode"] * 1e-3) / 1e9
        p = m["p10_med_p90_us"]
        print(f"| config {cfg} (x{m['R']} layers) | {wl0.batch} | {'f16' if wl0.dtype == 0 else 'bf16'} | {m['launches']} | "
              f"{m['bytes']['total'] / 1e6:.1f} | {m['ms'] * 1e3:.1f}; {p[0]:.1f}/{p[1]:.1f}/{p[2]:.1f} | {gb:.0f} | "
              f"{100 * gb / HBM_PEAK_GBPS:.1f} | {m['ms_decode'] * 1e3:.1f} | {dgb:.0f} | {cb['us_per_step']:.0f} ({cb['cores']}) |",
              flush=True)
        del insts
        torch.cuda.empty_cache()
    # dense reference through the same kernels: budget >= context on the headline cache
    wl0, insts, ub = make_instances(3, budget=131072, rotate=2)
    m = measure(wl0, insts, ub, 50, 5, stages=False)
    dgb = m["bytes"]["decode"] / (m["ms_decode"] * 1e-3) / 1e9
    print(f"| config 3, budget = context (dense read of 512 MiB) | 1 | f16 | {m['launches']} | {m['bytes']['total'] / 1e6:.1f} | "
          f"{m['ms'] * 1e3:.1f} | {m['bytes']['total'] / (m['ms'] * 1e-3) / 1e9:.0f} | "
          f"{100 * m['bytes']['total'] / (m['ms'] * 1e-3) / 1e9 / HBM_PEAK_GBPS:.1f} | {m['ms_decode'] * 1e3:.1f} | {dgb:.0f} | - |",
          flush=True)
    del insts
    torch.cuda.empty_cache()

    print("\nMax-min block representation (two INT4 vectors per block, twice the code stream), same workloads\n")
    print("| workload | useful MB/step | us/step | GB/s | planted-token recall: max-min / mean |")
    print("|---|---|---|---|---|", flush=True)
    for cfg in (1, 2, 3, 4):
        wl0, insts, ub = make_instances(cfg, block_repr=1)
        m = measure(wl0, insts, ub, args.steps, args.warmup, stages=False)
        dw = insts[0]
        dw.decode_fused()
        torch.cuda.synchronize()
        rec2 = O.planted_recall(wl0, dw.sel_idx.cpu().numpy(), dw.sel_cnt.cpu().numpy()) if wl0.planted else float("nan")
        r1 = O.decode_step(wl0, O.build_centroids(wl0, O.MEAN))
        rec1 = O.planted_recall(wl0, r1["sel_idx"], r1["sel_cnt"]) if wl0.planted else float("nan")
        gb = m["bytes"]["total"] / (m["ms"] * 1e-3) / 1e9
        print(f"| config {cfg} | {m['bytes']['total'] / 1e6:.1f} | {m['ms'] * 1e3:.1f} | {gb:.0f} | {rec2:.3f} / {rec1:.3f} |",
              flush=True)
        del insts, dw
        torch.cuda.empty_cache()

    print("\nPer-query-head selection (every query head ranks blocks by its own score and reads the rows of its own "
          "list: G times the code scans and up to G times the K/V rows; one centroid store per KV head), same workloads\n")
    print("| workload | launches/step | useful MB/step | us/step | GB/s | planted-token recall: per query head / per group |")
    print("|---|---|---|---|---|---|", flush=True)
    for cfg in (1, 2, 3, 4):
        wl0, insts, ub = make_instances(cfg, selection=1)
        m = measure(wl0, insts, ub, args.steps, args.warmup, stages=False)
        dw = insts[0]
        dw.decode_fused()
        torch.cuda.synchronize()
        if wl0.planted:
            view = O.per_query_head_view(wl0, caches=False)
            recq = O.planted_recall(view, dw.sel_idx.cpu().numpy(), dw.sel_cnt.cpu().numpy())
            r1 = O.decode_step(wl0, O.build_centroids(wl0, O.MEAN))
            recg = O.planted_recall(wl0, r1["sel_idx"], r1["sel_cnt"])
        else:
            recq = recg = float("nan")
        gb = m["bytes"]["total"] / (m["ms"] * 1e-3) / 1e9
        print(f"| config {cfg} | {m['launches']} | {m['bytes']['total'] / 1e6:.1f} | {m['ms'] * 1e3:.1f} | {gb:.0f} | "
              f"{recq:.3f} / {recg:.3f} |", flush=True)
        del insts, dw
        torch.cuda.empty_cache()

    print("\nGroup-maximum score (one selection per KV head, ranked by the maximum over its query heads of q . c^ "
          "instead of their sum: G integer dots per block and the heads' zero-point terms), same workloads\n")
    print("| workload | launches/step | useful MB/step | us/step | GB/s | planted-token recall: group maximum / group sum |")
    print("|---|---|---|---|---|---|", flush=True)
    for cfg in (1, 2, 3, 4):
        wl0, insts, ub = make_instances(cfg, selection=2)
        m = measure(wl0, insts, ub, args.steps, args.warmup, stages=False)
        dw = insts[0]
        dw.decode_fused()
        torch.cuda.synchronize()
        if wl0.planted:
            recm = O.planted_recall(wl0, dw.sel_idx.cpu().numpy(), dw.sel_cnt.cpu().numpy())
            r1 = O.decode_step(wl0, O.build_centroids(wl0, O.MEAN))
            recg = O.planted_recall(wl0, r1["sel_idx"], r1["sel_cnt"])
        else:
            recm = recg = float("nan")
        gb = m["bytes"]["total"] / (m["ms"] * 1e-3) / 1e9
        print(f"| config {cfg} | {m['launches']} | {m['bytes']['total'] / 1e6:.1f} | {m['ms'] * 1e3:.1f} | {gb:.0f} | "
              f"{recm:.3f} / {recg:.3f} |", flush=True)
        del insts, dw
        torch.cuda.empty_cache()

    print("\nStore maintenance while decoding (absb_append_token: one new token per request folded into the store, "
          "no rebuild) next to a full rebuild (absb_build_centroids)\n")
    print("| workload | segments | append us/call (back-to-back calls from Python: the host's call rate, the kernel "
          "itself takes ~3 us) | rebuild us/call | after 256 appended tokens: values of completed "
          "blocks outside the frozen ranges (the re-ranging signal) |")
    print("|---|---|---|---|---|", flush=True)
    from paper_2605_12110_amd.device import DeviceWorkload
    for cfg in (3, 4):
        import copy
        full = synth_workload(cfg)
        grow = 256
        wl0 = copy.copy(full)                       # the same caches, `grow` tokens before their final lengths
        wl0.seq_lens = full.seq_lens - grow
        dw = DeviceWorkload(wl0, cap_lens=full.seq_lens)
        dw.build()
        dw.tail_init()
        for t in range(1, grow + 1):                # real growth: ranges frozen at the build above
            dw.set_lens(wl0.seq_lens + t)
            dw.append_token()
        outside = int(dw.clamped.sum().item())
        bs = np.asarray(dw.block_size, dtype=np.int64)[None, :]
        closed = int((full.seq_lens.astype(np.int64)[:, None] // bs - wl0.seq_lens.astype(np.int64)[:, None] // bs).sum())
        ms_app, _ = time_loop(lambda i: dw.append_token(), 10, 100)      # the same token again and again: timing only
        ms_bld, _ = time_loop(lambda i: dw.build(), 2, 10)
        print(f"| config {cfg} | {dw.nseg} | {ms_app * 1e3:.1f} | {ms_bld * 1e3:.1f} | {outside} of {closed * 128} "
              f"({100.0 * outside / max(closed * 128, 1):.2f} %) in {closed} blocks |", flush=True)
        del dw
        torch.cuda.empty_cache()

    print(f"\nStreaming-read ceiling measured in this run (absb_stream_read, 2 GiB, 128-bit loads): "
          f"{stream_read_ceiling():.0f} GB/s of {HBM_PEAK_GBPS:.0f} GB/s published peak.")
    print("\nConfig 5 sweep (batch 4, context 65536, fp16): uniform block 16 vs adaptive per-head sizes\n")
    print("| blocks | budget | us/step | GB/s | planted-token recall | attention recall (mean) | max abs err vs dense | "
          "rel L2 err vs dense |")
    print("|---|---|---|---|---|---|---|---|", flush=True)
    for label, ublock in (("uniform 16", 16), ("seeded random draw per head", None)):
        for T in (1024, 2048, 4096, 8192):
            wl0, insts, ub = make_instances(5, budget=T, uniform_block=ublock, rotate=0)
            m = measure(wl0, insts, ub, args.steps, args.warmup, stages=False)
            dw = insts[0]
            dw.decode_fused()
            torch.cuda.synchronize()
            sel, cnt = dw.sel_idx.cpu().numpy(), dw.sel_cnt.cpu().numpy()
            got = dw.out_f32().astype(np.float64)
            dense, _ = O.dense_attention(wl0)
            rec_p = O.planted_recall(wl0, sel, cnt)
            rec_a = float(O.attention_recall(wl0, sel, cnt).mean())
            err = float(np.abs(got - dense).max())
            rel = float(np.linalg.norm(got - dense) / np.linalg.norm(dense))
            gb = m["bytes"]["total"] / (m["ms"] * 1e-3) / 1e9
            print(f"| {label} {wl0.block_size.tolist()} | {T} | {m['ms'] * 1e3:.1f} | {gb:.0f} | {rec_p:.3f} | {rec_a:.3f} | "
                  f"{err:.3e} | {rel:.3e} |", flush=True)
            del insts, dw
            torch.cuda.empty_cache()
    return rows


def run_calibration(args):
    """Sec. 3.2 on synthetic inputs: calibrate per-head block sizes on one set of samples, then compare
    the recall of the assignment with uniform sizes on held-out samples (markdown out)."""
    import torch
    from paper_2605_12110_amd import absb, calibrate, synth
    cand = calibrate.DEFAULT_CANDIDATES
    roles = (1, 1, 4, 4, 16, 16, 64, 64)          # run length of the heavy tokens per KV head: fixed head roles
    L, T = 32768, 1024

    def sample(seed):
        return synth.make_workload(5, batch=1, context=L, budget=T, seed=seed, run_lengths=roles)

    print(f"Calibration inputs: config-5 recipe, batch 1, context {L}, budget {T} tokens, fp16; heavy tokens of KV head h "
          f"sit in runs of {list(roles)} consecutive positions in every sample (head roles are a property of the "
          f"'model'); 8 calibration samples (seeds 300-307), 4 held-out samples (seeds 400-403).\n")
    t0 = time.perf_counter()
    per_sample = np.concatenate([calibrate.measure_recall(sample(300 + i), cand) for i in range(8)])
    torch.cuda.synchronize()
    print(f"Recall(h, B), mean over the calibration samples ({time.perf_counter() - t0:.1f} s for 8 samples x "
          f"{len(cand)} candidates, generation included):\n")
    _, mean = absb.absb_assign_block_sizes(per_sample, cand, 1.0)
    print("| KV head (run length) | " + " | ".join(f"B={b}" for b in cand) + " |")
    print("|---|" + "---|" * len(cand))
    for h in range(8):
        print(f"| {h} ({roles[h]}) | " + " | ".join(f"{mean[h, k]:.3f}" for k in range(len(cand))) + " |")
    _, held = absb.absb_assign_block_sizes(np.concatenate([calibrate.measure_recall(sample(400 + i), cand) for i in range(4)]),
                                           cand, 1.0)                 # the library's means over the held-out samples: [Hkv, cand]
    print("\nEq. (2) assignments and their recall on the held-out samples (mean over heads), against uniform sizes:\n")
    print("| assignment | block sizes | mean block size | blocks per 1K tokens (mean over heads) | held-out recall |")
    print("|---|---|---|---|---|")
    for k, b in enumerate(cand):
        print(f"| uniform | {b} | {b} | {1024 / b:.1f} | {held[:, k].mean():.3f} |")
    for tau in (0.98, 0.9, 0.8, 0.7, 0.6):
        sizes, _ = absb.absb_assign_block_sizes(per_sample, cand, tau)
        idx = [cand.index(int(s)) for s in sizes]
        rec = float(np.mean([held[h, idx[h]] for h in range(8)]))
        print(f"| Eq. (2), tau = {tau} | {sizes.tolist()} | {float(np.mean(sizes)):.1f} | "
              f"{float(np.mean(1024 / sizes)):.1f} | {rec:.3f} |", flush=True)

    # the same assignments timed: config-5 shape (batch 4, context 65536) with the head roles above, a
    # held-out seed, cold caches; quality against dense attention over the whole context from the oracle
    from oracle import oracle as O
    print("\nTimed A/B on the config-5 shape (batch 4, context 65536, fp16, head roles as above, seed 500): the step with "
          "calibrated sizes against uniform sizes, same budget; recall and error against dense attention\n")
    print("| assignment | block sizes | budget | us/step | useful MB/step | planted-token recall | attention recall (mean) | "
          "rel L2 err vs dense |")
    print("|---|---|---|---|---|---|---|---|", flush=True)
    assignments = [("uniform 16", [16] * 8), ("uniform 32", [32] * 8)]
    for tau in (0.9, 0.8, 0.7, 0.6):
        sizes, _ = absb.absb_assign_block_sizes(per_sample, cand, tau)
        if [int(x) for x in sizes] not in [a[1] for a in assignments]:
            assignments.append((f"Eq. (2), tau = {tau}", [int(x) for x in sizes]))
    for Tb in (1024, 4096):
        dense = None
        for label, sizes in assignments:
            wl0, insts, ub = make_instances(5, budget=Tb, seed=500, run_lengths=roles, head_block_sizes=sizes)
            m = measure(wl0, insts, ub, args.steps, args.warmup, stages=False)
            dw = insts[0]
            dw.decode_fused()
            torch.cuda.synchronize()
            sel, cnt = dw.sel_idx.cpu().numpy(), dw.sel_cnt.cpu().numpy()
            got = dw.out_f32().astype(np.float64)
            if dense is None:
                dense, _ = O.dense_attention(wl0)
            rel = float(np.linalg.norm(got - dense) / np.linalg.norm(dense))
            print(f"| {label} | {sizes} | {Tb} | {m['ms'] * 1e3:.1f} | {m['bytes']['total'] / 1e6:.1f} | "
                  f"{O.planted_recall(wl0, sel, cnt):.3f} | {float(O.attention_recall(wl0, sel, cnt).mean()):.3f} | "
                  f"{rel:.3e} |", flush=True)
            del insts, dw
            torch.cuda.empty_cache()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--config", type=int, default=3, help="workload recipe 1..5 (3 = headline)")
    ap.add_argument("--rotate", type=int, default=0,
                    help="resident copies cycled through (0 = auto: enough that a rotation touches 2 x the last-level cache)")
    ap.add_argument("--context", type=int, default=None)
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--budget", type=int, default=None)
    ap.add_argument("--select", choices=("group", "per-query-head", "group-max"), default="group",
                    help="who shares a selection: the query heads of a KV head, ranked by the sum of their scores "
                         "(default) or by their maximum, or nobody (one selection per query head)")
    ap.add_argument("--repr", choices=("mean", "minmax"), default="mean",
                    help="block representation: mean pooling (headline) or channel-wise maxima and minima")
    ap.add_argument("--form", type=int, default=0, choices=(0, 1, 2, 3),
                    help="how absb_decode_fused is enqueued (absb_step_form): 0 = the library's choice by shape "
                         "(default), 1 = pipelined one-launch step, 2 = one-launch step of units, 3 = one launch per stage")
    ap.add_argument("--split-tokens", type=int, default=0, help="absb_launch_opts.split_tokens (0 = the library's choice)")
    ap.add_argument("--unit-tokens", type=int, default=0, help="absb_launch_opts.unit_tokens (0 = the library's choice)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--matrix", action="store_true", help="run all configurations and the config-5 sweep; markdown out")
    ap.add_argument("--calibrate", action="store_true",
                    help="per-head block-size calibration (Eq. 2) on synthetic samples, with held-out validation; markdown out")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="run one device-to-device copy of this many MiB first (a kernel of known traffic, for "
                         "scaling hardware byte counters collected with rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_12110_amd import absb, synth
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

    if args.matrix:
        run_matrix(args)
        return
    if args.calibrate:
        run_calibration(args)
        return

    block_repr = 1 if args.repr == "minmax" else 0
    selection = {"group": 0, "per-query-head": 1, "group-max": 2}[args.select]
    wl0, insts, ub = make_instances(args.config, context=args.context, batch=args.batch, budget=args.budget,
                                    rotate=args.rotate, block_repr=block_repr, selection=selection,
                                    opts=dict(step_form=args.form, split_tokens=args.split_tokens, unit_tokens=args.unit_tokens))
    m = measure(wl0, insts, ub, args.steps, args.warmup, stages=True, percentiles=True)
    ms, R = m["ms"], m["R"]
    gbps = ub["total"] / (ms * 1e-3) / 1e9
    dec_gbps = ub["decode"] / (m["ms_decode"] * 1e-3) / 1e9
    ceiling = stream_read_ceiling()
    wl = wl0
    headline = (args.config == 3 and args.context is None and args.batch is None and args.budget is None
                and block_repr == 0 and args.select == "group")
    form_name = {absb.STEP_PIPELINED: "pipelined (one launch)", absb.STEP_UNITS: "units (one launch)",
                 absb.STEP_PER_STAGE: "per stage (three launches)"}[m["form"]]
    stages = {k: round(v, 3) for k, v in m["stages"].items()}
    if headline:
        # the same attention kernel on a budget that covers the context: a dense read of the layer's 512 MiB
        d_wl, d_insts, d_ub = make_instances(3, budget=int(wl.seq_lens.max()), rotate=2)
        for dw in d_insts:
            dw.batch.opts.counters_zero = 1
        d_ms = time_graph(lambda i: d_insts[i % 2].sparse_decode(), 2, 4, 20)
        stages["dense_read_us"] = round(d_ms * 1e3, 2)
        stages["dense_read_gbps"] = round(d_ub["decode"] / (d_ms * 1e-3) / 1e9, 1)
        del d_insts
        torch.cuda.empty_cache()
    result = {
        "metric": METRIC,
        "value": round(gbps, 2),
        "unit": "GB/s",
        "us_per_step": round(ms * 1e3, 3),
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
                        f"block sizes {wl.block_size.tolist()}, budget {int(wl.budget.max())} tokens, "
                        f"{args.repr} pooling, selection per {'query head' if args.select == 'per-query-head' else 'KV head'}"
                        f"{' (group maximum)' if args.select == 'group-max' else ''}",
            "entry_point": "absb_decode_fused",
            "step_form": form_name,
            "launches_per_step": m["launches"],
            "timing": "the timed steps captured into HIP graphs and replayed between two events on the launch stream",
            "resident_copies_rotated": R,
            "bytes_touched_per_rotation": int(R * ub["total"]),
            "cache_state": f"cold: {R} copies x {ub['total'] / 1e6:.1f} MB touched per step = "
                           f"{R * ub['total'] / LAST_LEVEL_CACHE_BYTES:.1f} x the 256 MB last-level cache between two visits of a copy",
            "resident_kv_bytes": int(sum(i.k_cache.numel() * 2 * 2 for i in insts)),
            "useful_bytes_per_step": {k: int(v) for k, v in ub.items()},
            "fraction_of_hbm_peak": round(gbps / HBM_PEAK_GBPS, 4),
            "eager_us_per_step": round(m["ms_eager"] * 1e3, 3),
            "host_wall_us_per_step_eager": round(m["wall_ms"] * 1e3, 2),
            "eager_us_per_step_p10_median_p90": [round(x, 2) for x in m["p10_med_p90_us"]],
            "stages": stages,
        },
    }
    if m["launches"] == 1:
        # the step is one launch: the dominant kernel is the step itself
        kern = "fused_step_kernel" if m["form"] == absb.STEP_PIPELINED else "step_kernel"
        result["roofline"] = {
            "bound": "hbm",
            "kernel": f"{kern} (one absb_decode_fused call = one launch: estimation, selection, attention)",
            "achieved": round(gbps, 2),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(gbps / HBM_PEAK_GBPS, 4),
            "algorithmic_bytes_per_launch": int(ub["total"]),
            "us_per_launch": round(ms * 1e3, 3),
            "traffic": measured_traffic(kern) if headline else None,
            "stream_read_ceiling": round(ceiling, 1),
            "frac_of_stream_read_ceiling": round(gbps / ceiling, 4),
        }
    else:
        result["roofline"] = {
            "bound": "hbm",
            # the timed unit is the entry point absb_sparse_decode with the split counters known to
            # be zero: exactly one launch of the attention kernel per call, on the fused step's selection
            "kernel": "decode_kernel (one absb_sparse_decode call = one launch)",
            "achieved": round(dec_gbps, 2),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(dec_gbps / HBM_PEAK_GBPS, 4),
            "algorithmic_bytes_per_launch": int(ub["decode"]),
            "us_per_launch": round(m["ms_decode"] * 1e3, 3),
            # counted by rocprofv3 --pmc on these very kernel sources (else null): see profiles/
            "traffic": measured_traffic("decode_kernel") if headline else None,
            # practical ceiling measured in this run: a plain 128-bit-load read of 2 GiB
            "stream_read_ceiling": round(ceiling, 1),
            "frac_of_stream_read_ceiling": round(dec_gbps / ceiling, 4),
        }
    if not args.no_cpu_baseline:
        cb = cpu_baseline(wl0, ub, block_repr=block_repr, check=insts, selection=selection)
        result["verified"] = cb.pop("verified")
        result["cpu_baseline"] = cb
    print(json.dumps(result))


if __name__ == "__main__":
    main()
