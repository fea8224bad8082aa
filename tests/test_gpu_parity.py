"""GPU parity: every stage of the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.  Integer results (codes, scores, selected block indices) must be
bit-exact; attention outputs must be within max-abs 2e-3 (fp16) / 1e-2 (bf16) of the fp64 oracle.
"""
import sys
import time

import numpy as np
import pytest

from oracle import oracle as O
from paper_2605_12110_amd import synth

pytestmark = pytest.mark.gpu

TOL = {synth.F16: 2e-3, synth.BF16: 1e-2}
LSE_TOL = 1e-4      # binary32 sums of the unrounded weights: measured <= 2e-6


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _dev(wl, **kw):
    import torch
    from paper_2605_12110_amd.device import DeviceWorkload
    assert torch.cuda.is_available()
    return DeviceWorkload(wl, **kw)


def _sync():
    import torch
    torch.cuda.synchronize()


from contextlib import contextmanager


@contextmanager
def _opts(dw, **kw):
    """Launch options of the holder's batch (absb_launch_opts) for the calls inside the block."""
    old = {k: getattr(dw.batch.opts, k) for k in kw}
    for k, v in kw.items():
        setattr(dw.batch.opts, k, v)
    try:
        yield
    finally:
        for k, v in old.items():
            setattr(dw.batch.opts, k, v)


FORMS = {1: "pipelined", 2: "units", 3: "per stage"}      # absb_step_form


def _check_out(dw, want_out, want_lse, what):
    _sync()
    got = dw.out_f32().astype(np.float64)
    err = np.abs(got - want_out).max()
    lse = dw.lse.cpu().numpy().astype(np.float64)
    fin = np.isfinite(want_lse)
    lerr = np.abs(lse[fin] - want_lse[fin]).max() if fin.any() else 0.0
    _say(f"    {what}: max|out-oracle| = {err:.3e} (tol {TOL[dw.wl.dtype]:.0e}), max|lse-oracle| = {lerr:.3e}")
    assert np.isfinite(got).all()
    assert err <= TOL[dw.wl.dtype], what
    assert lerr <= LSE_TOL, what
    assert np.array_equal(np.isneginf(lse), np.isneginf(want_lse))


def run_all_stages(wl, name, block_repr=O.MEAN, per_query_head=False, group_max=False):
    """Stage by stage (each GPU stage fed the oracle's inputs), then the fused call end to end."""
    _say(f"[case {name}] repr={block_repr} Bt={wl.batch} Hq={wl.num_q_heads} Hkv={wl.num_kv_heads} P={wl.page_size} "
         f"L={wl.seq_lens.tolist()[:4]}.. B={wl.block_size.tolist()} T={wl.budget.tolist()[:4]}.. dtype={wl.dtype}")
    t0 = time.time()
    st = O.build_centroids(wl, block_repr)
    if per_query_head:
        # the reference is the method on the model in which every query head is its own group; the
        # library keeps ONE store per KV head (st) and must reproduce that model's scores (same flat
        # layout: the G copies of a store segment side by side), lists and outputs
        view = O.per_query_head_view(wl)
        ref = O.decode_step(view, O.build_centroids(view, block_repr), sel_stride=None)
    else:
        ref = O.decode_step(wl, st, sel_stride=None, group_max=group_max)
    _say(f"    oracle: build+step {time.time() - t0:.2f}s, centroids={int(st.off[-1])}, per_query_head={per_query_head}")
    from paper_2605_12110_amd import absb as _absb
    dw = _dev(wl, block_repr=block_repr,      # the two enumerations agree: 0 mean, 1 maxima and minima
              selection=_absb.SELECT_PER_QUERY_HEAD if per_query_head else
              _absb.SELECT_GROUP_MAX if group_max else _absb.SELECT_GROUP)
    assert np.array_equal(dw.plan.cent_off.astype(np.int64), st.off)
    K = dw.sel_stride
    assert K == int(ref["sel_cnt"].max())

    # a0 build: bit-exact codes and parameters
    dw.build(); _sync()
    codes = dw.codes.cpu().numpy()
    assert np.array_equal(dw.qscale.cpu().numpy(), st.qscale), "qscale"
    assert np.array_equal(dw.qmin.cpu().numpy(), st.qmin), "qmin"
    nbad = int((codes != st.codes).sum())
    assert nbad == 0, f"{nbad} code bytes differ"
    _say("    build: codes/qscale/qmin bit-exact")

    # a1 score on the oracle's store
    dw.load_store(st.codes, st.qscale, st.qmin)
    dw.score(); _sync()
    assert np.array_equal(dw.score_exp.cpu().numpy(), ref["score_exp"]), "score exponent"
    assert np.array_equal(dw.scores.cpu().numpy(), ref["scores"]), "scores"
    _say("    score: int32 scores bit-exact")

    # a2 top-k on the oracle's scores
    import torch
    dw.scores.copy_(torch.from_numpy(ref["scores"]))
    dw.sel_idx.fill_(-7); dw.sel_cnt.fill_(-7)
    dw.topk(); _sync()
    assert np.array_equal(dw.sel_cnt.cpu().numpy(), ref["sel_cnt"]), "sel_cnt"
    assert np.array_equal(dw.sel_idx.cpu().numpy(), ref["sel_idx"][:, :K]), "sel_idx"
    _say("    topk: indices bit-exact")

    # a3-a5 sparse decode on the oracle's selection
    dw.sel_idx.copy_(torch.from_numpy(np.ascontiguousarray(ref["sel_idx"][:, :K])))
    dw.sel_cnt.copy_(torch.from_numpy(ref["sel_cnt"]))
    dw.out.fill_(float("nan")); dw.lse.fill_(float("nan"))
    dw.sparse_decode()
    _check_out(dw, ref["out"], ref["lse"], "sparse_decode")

    # the whole step from the GPU-built store
    dw.build()
    dw.sel_idx.fill_(-7); dw.sel_cnt.fill_(-7); dw.out.fill_(float("nan")); dw.lse.fill_(float("nan"))
    dw.scribble(0x5A)
    dw.decode_fused()
    _check_out(dw, ref["out"], ref["lse"], "decode_fused")
    assert np.array_equal(dw.sel_cnt.cpu().numpy(), ref["sel_cnt"])
    assert np.array_equal(dw.sel_idx.cpu().numpy(), ref["sel_idx"][:, :K])
    # and again without asking for the selection, different workspace poison: same bits out
    first = dw.out.cpu().numpy().copy() if dw.out.dtype == torch.float16 else dw.out.float().cpu().numpy().copy()
    dw.scribble(0xC3)
    dw.decode_fused(want_sel=False); _sync()
    second = dw.out.cpu().numpy() if dw.out.dtype == torch.float16 else dw.out.float().cpu().numpy()
    assert np.array_equal(first, second), "fused output depends on workspace contents or is not deterministic"
    # every way of enqueueing the step, forced (the default picks one by shape): two one-launch forms
    # and one launch per stage (which needs no cleared counters).  Same selection from all; outputs
    # within tolerance of the oracle.  Each form is deterministic; they sum in different orders (the
    # pipelined form's attention reads the selection in the order its members were found)
    from paper_2605_12110_amd import absb
    outs = {}
    for mode in (1, 2, 3):
        with _opts(dw, step_form=mode):
            dw.sel_idx.fill_(-7); dw.sel_cnt.fill_(-7); dw.out.fill_(float("nan")); dw.lse.fill_(float("nan"))
            if mode == 3:
                dw.workspace.fill_(0x3C)
            else:
                dw.scribble(0x3C)
            dw.decode_fused()
            _check_out(dw, ref["out"], ref["lse"], f"decode_fused, {FORMS[mode]}")
        outs[mode] = dw.out.cpu().numpy() if dw.out.dtype == torch.float16 else dw.out.float().cpu().numpy()
        assert np.array_equal(dw.sel_cnt.cpu().numpy(), ref["sel_cnt"]), FORMS[mode]
        assert np.array_equal(dw.sel_idx.cpu().numpy(), ref["sel_idx"][:, :K]), FORMS[mode]
        if mode != 3:
            assert dw.status() == 0, FORMS[mode]
            # and once more without asking for the list: same bits (nothing depends on the workspace's contents)
            with _opts(dw, step_form=mode):
                dw.scribble(0xC5)
                dw.decode_fused(want_sel=False); _sync()
            again = dw.out.cpu().numpy() if dw.out.dtype == torch.float16 else dw.out.float().cpu().numpy()
            assert np.array_equal(outs[mode], again), f"{FORMS[mode]}: not deterministic, or the list request changes the output"
    assert np.array_equal(first, outs[absb.absb_step_form_used(dw.layer, dw.batch)]), "default form"
    dw.check_device_contents(lists=True)      # the holder's host-side bounds checks agree with all of that
    dw.scribble(0x99)     # the stand-alone stages do not keep the other counters: clear them again
    _say("    fused: selection bit-exact in every enqueue form, outputs within tolerance, deterministic")
    return dw, st, ref


# ------------------------------------------------------------------ small cases: several tiles, ragged tails
@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
def test_ragged_small_batch(dtype):
    wl = synth.tiny_workload(seed=21, dtype=dtype, Bt=3, Hq=8, Hkv=2, P=16, seq_lens=(37, 64, 1301),
                             block_size=(8, 32), budget=(16, 24, 400))
    run_all_stages(wl, f"ragged dtype={dtype}")


def test_group_of_five_and_blocks_larger_than_a_page():
    wl = synth.tiny_workload(seed=22, dtype=synth.BF16, Bt=2, Hq=20, Hkv=4, P=16, seq_lens=(999, 2500),
                             block_size=(128, 8, 64, 16), budget=(300, 520))
    run_all_stages(wl, "G=5, B>P")


@pytest.mark.parametrize("G", [1, 2, 3, 6, 7, 8])
def test_other_group_sizes(G):
    wl = synth.tiny_workload(seed=23 + G, dtype=synth.F16, Bt=1, Hq=2 * G, Hkv=2, P=64, seq_lens=(777,),
                             block_size=(16, 128), budget=(200,))
    run_all_stages(wl, f"G={G}")


def test_config1_full():
    run_all_stages(synth.make_workload(1), "config1")


def test_config2_scaled():
    run_all_stages(synth.make_workload(2, context=8192, batch=3, budget=1024), "config2 (8K ctx, batch 3)")


def test_config4_scaled_mixed_lengths():
    run_all_stages(synth.make_workload(4, context=16384, batch=5), "config4 (<=16K ctx, batch 5)")


def test_config5_uniform16_scaled():
    run_all_stages(synth.make_workload(5, context=16384, batch=2, uniform_block=16, budget=2048), "config5-U")


# ------------------------------------------------------------------ full-size cases
def test_config3_full_headline():
    """128K context, batch 1: the configuration the benchmark times."""
    dw, st, ref = run_all_stages(synth.make_workload(3), "config3 full (128K)")
    # every selected block holds the budget: K_s * B_h = 4096
    assert np.all(ref["sel_cnt"] * dw.wl.block_size == 4096)


def test_config2_full():
    run_all_stages(synth.make_workload(2), "config2 full (8 x 32K)")


def test_config4_full_mixed_batch():
    """16 requests of 8K..128K tokens, 40 query / 8 KV heads (group of 5), bf16, budget 3 % of each context."""
    run_all_stages(synth.make_workload(4), "config4 full (16 mixed lengths)")


def test_config5_full_adaptive():
    run_all_stages(synth.make_workload(5), "config5 full (4 x 64K, adaptive)")


# ------------------------------------------------------------------ edge cases
def test_budget_covering_the_context_is_dense_attention():
    wl = synth.tiny_workload(seed=31, dtype=synth.F16, Bt=2, Hq=8, Hkv=2, P=16, seq_lens=(300, 129),
                             block_size=(8, 64), budget=(10 ** 6, 129))
    dw, st, ref = run_all_stages(wl, "dense")
    dense, dense_lse = O.dense_attention(wl)
    dw.decode_fused()
    _check_out(dw, dense, dense_lse, "fused vs dense oracle")


def test_single_token_context_and_single_block_budget():
    wl = synth.tiny_workload(seed=32, dtype=synth.BF16, Bt=2, Hq=4, Hkv=2, P=16, seq_lens=(1, 50),
                             block_size=(8, 16), budget=(1, 1))
    dw, st, ref = run_all_stages(wl, "L=1 / K=1")
    assert list(ref["sel_cnt"]) == [1, 1, 1, 1]
    # L = 1: the output is exactly that token's value
    v = wl.value_rows(0, 0)[0]
    assert np.array_equal(dw.out_f32()[0, 0], v)


def test_all_equal_scores_pick_lowest_indices():
    import torch
    wl = synth.tiny_workload(seed=33, Bt=1, Hq=4, Hkv=2, P=16, seq_lens=(4096,), block_size=(8, 16), budget=(800,))
    dw = _dev(wl)
    dw.scores.fill_(12345)
    dw.topk(); _sync()
    cnt = dw.sel_cnt.cpu().numpy()
    idx = dw.sel_idx.cpu().numpy()
    assert list(cnt) == [100, 50]
    assert np.array_equal(idx[0, :100], np.arange(100)) and np.array_equal(idx[1, :50], np.arange(50))
    assert np.all(idx[1, 50:] == -1)
    # extreme values and heavy ties against the oracle
    rng = np.random.default_rng(0)
    sc = rng.choice(np.array([-2 ** 31, -1, 0, 1, 2 ** 31 - 1], dtype=np.int64), size=dw.plan.total_centroids)
    sc = sc.astype(np.int32)
    dw.scores.copy_(torch.from_numpy(sc))
    dw.topk(); _sync()
    want_idx, want_cnt = O.topk(wl, dw.plan.cent_off.astype(np.int64), sc, sel_stride=dw.sel_stride)
    assert np.array_equal(dw.sel_idx.cpu().numpy(), want_idx) and np.array_equal(dw.sel_cnt.cpu().numpy(), want_cnt)


def test_decode_accepts_any_list_order_partial_last_block_and_empty_lists():
    import torch
    wl = synth.tiny_workload(seed=34, dtype=synth.F16, Bt=2, Hq=8, Hkv=2, P=16, seq_lens=(203, 77),
                             block_size=(8, 32), budget=(256, 256))      # lists below stay within K_s
    dw = _dev(wl)
    K = dw.sel_stride
    rng = np.random.default_rng(1)
    sel = np.full((4, K), -1, np.int32)
    cnt = np.zeros(4, np.int32)
    for s in range(4):
        b, h = divmod(s, 2)
        N = -(-int(wl.seq_lens[b]) // int(wl.block_size[h]))
        k = min(K, N, 1 + s)
        pick = rng.choice(N - 1, size=k - 1, replace=False).tolist() + [N - 1]   # always the partial last block
        rng.shuffle(pick)
        sel[s, :k] = pick
        cnt[s] = k
    cnt[2] = 0                                                                   # an empty selection
    sel[2, :] = -1
    want, want_lse = O.sparse_attention(wl, sel, cnt)
    dw.sel_idx.copy_(torch.from_numpy(sel)); dw.sel_cnt.copy_(torch.from_numpy(cnt))
    dw.out.fill_(float("nan")); dw.lse.fill_(float("nan"))
    dw.sparse_decode()
    _check_out(dw, want, want_lse, "arbitrary lists")
    G = wl.group
    assert not dw.out_f32()[1, 0:G].any() and np.all(np.isneginf(dw.lse.cpu().numpy()[1, 0:G]))


def test_split_shapes_do_not_change_the_selection_and_stay_within_tolerance():
    wl = synth.make_workload(1, context=8192, budget=2048)
    st = O.build_centroids(wl)
    ref = O.decode_step(wl, st)
    for split in (64, 128, 512, 1024):
        for form in (1, 3):
            dw = _dev(wl, opts=dict(split_tokens=split, step_form=form))
            dw.build()
            dw.decode_fused()
            _check_out(dw, ref["out"], ref["lse"], f"split_tokens={split}, {FORMS[form]}")
            assert np.array_equal(dw.sel_idx.cpu().numpy(), ref["sel_idx"][:, :dw.sel_stride])
    for unit in (64, 256, 1024):
        dw = _dev(wl, opts=dict(unit_tokens=unit, step_form=2))
        dw.build()
        dw.decode_fused()
        _check_out(dw, ref["out"], ref["lse"], f"unit_tokens={unit}, units")
        assert np.array_equal(dw.sel_idx.cpu().numpy(), ref["sel_idx"][:, :dw.sel_stride])
        assert dw.status() == 0
    for chunk in (64, 1024):
        dw = _dev(wl, opts=dict(score_chunk=chunk))
        dw.load_store(st.codes, st.qscale, st.qmin)
        dw.score(); _sync()
        assert np.array_equal(dw.scores.cpu().numpy(), ref["scores"])


def test_nonstandard_cache_strides_nhd_layout():
    """Token-major pages ([page][slot][head][d]) through the stride fields."""
    import torch
    from paper_2605_12110_amd import absb
    wl = synth.tiny_workload(seed=35, dtype=synth.F16, Bt=2, Hq=8, Hkv=2, P=16, seq_lens=(150, 90),
                             block_size=(8, 32), budget=(48, 48))
    st = O.build_centroids(wl)
    ref = O.decode_step(wl, st)
    dw = _dev(wl)
    # re-lay the caches as NHD on the device and point the layer's strides at that layout
    H, P, d = wl.num_kv_heads, wl.page_size, wl.head_dim
    dw.k_cache = dw.k_cache.permute(0, 2, 1, 3).contiguous()
    dw.v_cache = dw.v_cache.permute(0, 2, 1, 3).contiguous()
    dw.layer = absb.Layer(wl.num_q_heads, H, d, P, wl.dtype, wl.block_size, (P * H * d, d, H * d))
    dw.build(); _sync()
    assert np.array_equal(dw.codes.cpu().numpy(), st.codes)
    dw.decode_fused()
    _check_out(dw, ref["out"], ref["lse"], "NHD strides")
    assert np.array_equal(dw.sel_idx.cpu().numpy(), ref["sel_idx"][:, :dw.sel_stride])


def test_many_splits_per_segment_and_split_counters_left_at_zero():
    """More splits than one merge round trip covers; then the stand-alone attention call with the
    caller's promise that the split counters are zero (they are: every launch leaves them so, and
    a rebuild of the centroid store in between does not touch them)."""
    from paper_2605_12110_amd import absb
    wl = synth.make_workload(1, context=8192, budget=8192)       # every block selected: 8192 tokens per segment
    st = O.build_centroids(wl)
    ref = O.decode_step(wl, st)
    dw = _dev(wl, opts=dict(split_tokens=64, step_form=1))       # 128 splits per segment
    dw.build()
    dw.decode_fused()
    _check_out(dw, ref["out"], ref["lse"], "128 splits, fused")
    dw.build()
    with _opts(dw, counters_zero=1):
        for rep in range(3):
            dw.out.fill_(float("nan")); dw.lse.fill_(float("nan"))
            dw.sparse_decode()
            _check_out(dw, ref["out"], ref["lse"], f"128 splits, stand-alone call {rep}, counters promised zero")
    dw.workspace.fill_(0x5A)                                 # garbage counters: the default path clears them
    dw.out.fill_(float("nan")); dw.lse.fill_(float("nan"))
    dw.sparse_decode()
    _check_out(dw, ref["out"], ref["lse"], "128 splits, stand-alone call on a scribbled workspace")


def test_host_side_bounds_checks_of_the_holder_catch_bad_device_contents():
    """The debug aid that stands in for device-side asserts: planted violations are named on the host."""
    import torch
    wl = synth.tiny_workload(seed=61, Bt=2, Hq=8, Hkv=2, P=16, seq_lens=(100, 50), block_size=(8, 32), budget=(32, 32))
    dw = _dev(wl)
    dw.build(); dw.decode_fused(); _sync()
    dw.check_device_contents(lists=True)
    keep = dw.page_table.clone()
    dw.page_table[1, 2] = int(dw.k_cache.shape[0])               # one page past the cache
    with pytest.raises(AssertionError, match="page table of request 1"):
        dw.check_device_contents()
    dw.page_table.copy_(keep)
    dw.sel_idx[3, 0] = 10 ** 6
    with pytest.raises(AssertionError, match="sel_idx"):
        dw.check_device_contents(lists=True)
    dw.seq_lens[0] += 1
    with pytest.raises(AssertionError, match="seq_lens"):
        dw.check_device_contents()


def test_stream_read_helper_runs_and_leaves_its_sink_alone():
    import torch
    from paper_2605_12110_amd import absb
    buf = torch.arange(0, (1 << 20) + 48, dtype=torch.int32, device="cuda")   # a ragged tile count
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    absb.absb_stream_read(buf, sink)
    _sync()
    assert int(sink.item()) == 0
    with pytest.raises(absb.AbsbError):
        absb.absb_stream_read(buf.view(torch.uint8)[4:], sink)                # misaligned source


@pytest.mark.parametrize("kind", ["random", "few_values", "all_equal", "few_values_forced", "random_forced"])
def test_selection_at_the_largest_supported_segment(kind):
    """2^17 blocks in one segment (the selection kernel's capacity), two segments of different
    size side by side; heavy ties push the kernel onto its multi-digit path."""
    import torch
    from paper_2605_12110_amd import absb
    B = np.array([8, 16], np.int32)
    L = np.array([8 << 17], np.int32)                       # 131072 blocks of 8, 65536 blocks of 16
    T = np.array([160000], np.int32)                        # K = 20000 and 10000 blocks
    sink, recent = (1000, 40000) if kind.endswith("forced") else (0, 0)
    layer = absb.Layer(2, 2, 128, 64, synth.F16, B, (2 * 64 * 128, 64 * 128, 128), sink_tokens=sink,
                       recent_tokens=recent)
    dev = "cuda:0"
    batch = absb.Batch(seq_lens_host=L, budget_host=T, seq_lens=torch.from_numpy(L).to(dev),
                       page_table=None, budget=torch.from_numpy(T).to(dev), pt_stride=int(L[0]) // 64)
    plan = absb.absb_plan(layer, batch)
    off = plan.cent_off.astype(np.int64)
    assert off.tolist() == [0, 1 << 17, (1 << 17) + (1 << 16)]
    batch.cent_off = torch.from_numpy(plan.cent_off).to(dev)
    rng = np.random.default_rng(77)
    total = int(off[-1])
    if kind.startswith("random"):
        sc = rng.integers(-2 ** 31, 2 ** 31, size=total, dtype=np.int64)
    elif kind.startswith("few_values"):
        sc = rng.integers(-3, 4, size=total, dtype=np.int64) * 1000003
    else:
        sc = np.full(total, -17, np.int64)
    sc = sc.astype(np.int32)
    stride = plan.sel_stride
    assert stride == 20000
    sel_idx = torch.full((2, stride), -7, dtype=torch.int32, device=dev)
    sel_cnt = torch.full((2,), -7, dtype=torch.int32, device=dev)
    _say(f"[case top-k capacity/{kind}] blocks={np.diff(off).tolist()} K={[20000, 10000]}")
    absb.absb_topk(layer, batch, torch.from_numpy(sc).to(dev), sel_idx, sel_cnt, stride)
    _sync()
    want_idx, want_cnt = O.topk_raw(1, 2, off, B, T, sc, stride, L, sink, recent)
    assert np.array_equal(sel_cnt.cpu().numpy(), want_cnt) and want_cnt.tolist() == [20000, 10000]
    assert np.array_equal(sel_idx.cpu().numpy(), want_idx)


# ------------------------------------------------------------------ max-min block representation
@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
def test_minmax_ragged_small_batch(dtype):
    wl = synth.tiny_workload(seed=41, dtype=dtype, Bt=3, Hq=8, Hkv=2, P=16, seq_lens=(37, 64, 1301),
                             block_size=(8, 32), budget=(16, 24, 400))
    run_all_stages(wl, f"max-min ragged dtype={dtype}", O.MINMAX)


@pytest.mark.parametrize("G", [1, 5, 8])
def test_minmax_group_sizes_and_blocks_larger_than_a_page(G):
    wl = synth.tiny_workload(seed=42 + G, dtype=synth.BF16, Bt=2, Hq=4 * G, Hkv=4, P=16, seq_lens=(999, 2500),
                             block_size=(128, 8, 64, 16), budget=(300, 520))
    run_all_stages(wl, f"max-min G={G}, B>P", O.MINMAX)


def test_minmax_config1_full():
    run_all_stages(synth.make_workload(1), "max-min config1", O.MINMAX)


def test_minmax_config3_full_headline():
    run_all_stages(synth.make_workload(3), "max-min config3 (headline shape)", O.MINMAX)


def test_minmax_config4_scaled_mixed_lengths():
    run_all_stages(synth.make_workload(4, context=16384, batch=5), "max-min config4 (<=16K ctx, batch 5)", O.MINMAX)


# ------------------------------------------------------------------ calibration (Sec. 3.2)
def test_calibration_recall_and_assignment_match_the_oracle():
    """Recall(h, B) measured through the library (two log-sum-exp arrays per candidate) against the
    oracle's fp64 recall of the oracle's own selection, and Eq. (2) on both sides."""
    from paper_2605_12110_amd import absb, calibrate
    cand = (8, 16, 32, 64, 128)
    samples = [synth.make_workload(3, context=8192, budget=512, seed=100 + i) for i in range(3)]
    sizes, mean, per_sample = calibrate.calibrate(samples, cand, tau=0.6)
    want = np.empty((len(samples), samples[0].num_kv_heads, len(cand)))
    for i, wl in enumerate(samples):
        for k, B in enumerate(cand):
            wl_b = synth.make_workload(3, context=8192, budget=512, seed=100 + i, uniform_block=B)
            assert np.array_equal(wl_b.k_cache, wl.k_cache) and np.array_equal(wl_b.q, wl.q)
            r = O.decode_step(wl_b, O.build_centroids(wl_b))
            want[i, :, k] = O.head_recall(wl_b, r["sel_idx"], r["sel_cnt"]).mean(axis=0)
    err = np.abs(per_sample - want).max()
    _say(f"[case calibration] max |recall - oracle| = {err:.2e}; mean recall per head x candidate:\n{np.round(mean, 3)}")
    assert err <= 2e-3
    # the rule itself is integer work: identical on identical (float32) recalls
    o_sizes, o_mean = O.assign_block_sizes(per_sample.astype(np.float64), cand, 0.6)
    assert np.array_equal(sizes, o_sizes) and np.allclose(mean, o_mean, rtol=1e-15, atol=0)
    # and from the oracle's own recalls, wherever no mean sits within the recall tolerance of its threshold
    w_sizes, w_mean = O.assign_block_sizes(want, cand, 0.6)
    margin = np.abs(w_mean - 0.6 * w_mean[:, :1]).min(axis=1)
    safe = margin > 4e-3
    assert safe.any() and np.array_equal(sizes[safe], w_sizes[safe])
    assert len(set(w_sizes.tolist())) >= 3                   # the heads of this input do not all want the same size
    _say(f"    block sizes: library {sizes.tolist()}, oracle {w_sizes.tolist()} (compared on {int(safe.sum())} heads)")


# ------------------------------------------------------------------ forced sink / recent blocks
@pytest.mark.parametrize("sink,recent", [(1, 0), (0, 1), (64, 200), (5000, 5000)])
def test_forced_sink_and_recent_blocks(sink, recent):
    """Selection policy knob: blocks holding the first / last tokens always rank first.  Bit-exact
    selection against the oracle, attention within tolerance, through the stand-alone and fused calls."""
    wl = synth.tiny_workload(seed=51, dtype=synth.F16, Bt=3, Hq=8, Hkv=4, P=16, seq_lens=(37, 640, 2301),
                             block_size=(8, 32, 128, 16), budget=(16, 96, 400))
    st = O.build_centroids(wl)
    ref = O.decode_step(wl, st, sink_tokens=sink, recent_tokens=recent)
    plain = O.decode_step(wl, st)
    assert not np.array_equal(ref["sel_idx"], plain["sel_idx"])          # the knob changes something here
    dw = _dev(wl, sink_tokens=sink, recent_tokens=recent)
    K = dw.sel_stride
    _say(f"[case forced sink={sink} recent={recent}] K={K}")
    dw.load_store(st.codes, st.qscale, st.qmin)
    dw.score(); dw.topk(); _sync()
    assert np.array_equal(dw.sel_cnt.cpu().numpy(), ref["sel_cnt"])
    assert np.array_equal(dw.sel_idx.cpu().numpy(), ref["sel_idx"][:, :K])
    dw.build()
    dw.sel_idx.fill_(-7); dw.sel_cnt.fill_(-7)
    dw.decode_fused()
    _check_out(dw, ref["out"], ref["lse"], "decode_fused with forced blocks")
    assert np.array_equal(dw.sel_idx.cpu().numpy(), ref["sel_idx"][:, :K])


def test_forced_blocks_on_a_long_segment_with_many_tiles():
    wl = synth.make_workload(3, context=65536, budget=2048)              # up to 8192 blocks per segment
    st = O.build_centroids(wl)
    ref = O.decode_step(wl, st, sink_tokens=128, recent_tokens=1024)
    dw = _dev(wl, sink_tokens=128, recent_tokens=1024)
    dw.build()
    dw.decode_fused()
    _check_out(dw, ref["out"], ref["lse"], "forced blocks, 64K context")
    assert np.array_equal(dw.sel_idx.cpu().numpy(), ref["sel_idx"][:, :dw.sel_stride])
    # every segment holds its first block and its last ones
    sel, cnt = dw.sel_idx.cpu().numpy(), dw.sel_cnt.cpu().numpy()
    for s in range(8):
        B = int(wl.block_size[s])
        chosen = set(sel[s, :cnt[s]].tolist())
        want = set(range(-(-128 // B))) | set(range((65536 - 1024) // B, 65536 // B))
        assert (want <= chosen) if len(want) <= cnt[s] else (chosen <= want)


@pytest.mark.parametrize("Hkv,G", [(33, 2), (64, 1), (64, 8)])
def test_many_kv_heads(Hkv, G):
    """Head counts beyond the benchmark shapes, up to the 64 KV heads the head table holds."""
    rng = np.random.default_rng(Hkv * 10 + G)
    wl = synth.tiny_workload(seed=Hkv, dtype=synth.BF16 if G == 1 else synth.F16, Bt=2, Hq=Hkv * G, Hkv=Hkv, P=32,
                             seq_lens=(700, 65), block_size=rng.choice([8, 16, 32, 64, 128], size=Hkv).tolist(),
                             budget=(96, 2048))
    run_all_stages(wl, f"{Hkv} KV heads x {G}", group_max=G == 8)


@pytest.mark.parametrize("L,sizes,G,budget", [(1 << 20, (8, 128), 4, 8192), ((1 << 20) - 3, (8,), 1, 1 << 20)])
def test_one_million_token_context(L, sizes, G, budget):
    """The longest segment the selection holds (2^17 blocks of 8 tokens) through every stage and the
    fused step; the second case selects all of it (a dense read through a 131072-entry list)."""
    wl = synth.tiny_workload(seed=L % 1000, dtype=synth.F16, Bt=1, Hq=len(sizes) * G, Hkv=len(sizes), P=64,
                             seq_lens=(L,), block_size=sizes, budget=(budget,))
    run_all_stages(wl, f"context {L}, blocks {sizes}, budget {budget}")


@pytest.mark.parametrize("P", [2048, 65536])
def test_pages_much_larger_than_blocks(P):
    """Up to the largest page the plan accepts (65536 tokens): hundreds of blocks per page."""
    wl = synth.tiny_workload(seed=P, dtype=synth.BF16, Bt=2, Hq=6, Hkv=2, P=P, seq_lens=(P + 37, 700),
                             block_size=(8, 128), budget=(200, 1000), extra_pages=1)
    run_all_stages(wl, f"page size {P}")


def test_the_largest_number_of_segments():
    """65535 selection segments (the limit of the plan), each a short context: every stage and the
    fused step in all its forms."""
    rng = np.random.default_rng(65535)
    Bt = 13107
    lens = rng.integers(1, 200, size=Bt).tolist()
    wl = synth.tiny_workload(seed=65535, dtype=synth.F16, Bt=Bt, Hq=5, Hkv=5, P=16, seq_lens=lens,
                             block_size=(16, 16, 64, 8, 128), budget=rng.choice([1, 8, 64, 1000], size=Bt).tolist())
    run_all_stages(wl, "65535 segments")


def test_optional_outputs_may_be_left_out_and_lists_may_be_wider_than_needed():
    """lse, score_exp and the copies of the selection are optional (NULL); a list buffer wider than
    absb_plan's sel_stride is padded with -1 to its full width."""
    import torch
    from paper_2605_12110_amd import absb
    wl = synth.tiny_workload(seed=97, dtype=synth.F16, Bt=3, Hq=8, Hkv=2, P=16, seq_lens=(333, 2100, 64),
                             block_size=(8, 64), budget=(100, 512, 64))
    st = O.build_centroids(wl)
    ref = O.decode_step(wl, st)
    dw = _dev(wl)
    dw.build()
    absb.absb_score(dw.layer, dw.batch, dw.q, dw.codes, dw.qscale, dw.scores, None)
    wide = dw.sel_stride + 19
    sel = torch.full((dw.nsel, wide), -7, dtype=torch.int32, device=dw.device)
    cnt = torch.full((dw.nsel,), -7, dtype=torch.int32, device=dw.device)
    absb.absb_topk(dw.layer, dw.batch, dw.scores, sel, cnt, wide)
    _sync()
    assert np.array_equal(dw.scores.cpu().numpy(), ref["scores"])
    got = sel.cpu().numpy()
    assert np.array_equal(cnt.cpu().numpy(), ref["sel_cnt"])
    assert np.array_equal(got[:, :dw.sel_stride], ref["sel_idx"][:, :dw.sel_stride]) and np.all(got[:, dw.sel_stride:] == -1)
    dw.out.fill_(float("nan"))
    absb.absb_sparse_decode(dw.layer, dw.batch, dw.q, dw.k_cache, dw.v_cache, sel, cnt, wide, dw.out, None, dw.workspace)
    _sync()
    assert np.abs(dw.out_f32().astype(np.float64) - ref["out"]).max() <= TOL[wl.dtype]
    dw.scribble(0x21)
    dw.out.fill_(float("nan"))
    absb.absb_decode_fused(dw.layer, dw.batch, dw.q, dw.codes, dw.qscale, dw.k_cache, dw.v_cache, dw.out, None, None, None,
                           dw.workspace)
    _sync()
    assert np.abs(dw.out_f32().astype(np.float64) - ref["out"]).max() <= TOL[wl.dtype]
    assert dw.status() == 0


@pytest.mark.parametrize("scale", [0.02, 0.25, 1.0])
def test_caller_given_softmax_scale(scale):
    """absb_layer.sm_scale other than 1/sqrt(d): flat and very peaked softmax, stand-alone and fused."""
    import torch
    wl = synth.tiny_workload(seed=96, dtype=synth.BF16, Bt=2, Hq=10, Hkv=2, P=16, seq_lens=(900, 130),
                             block_size=(16, 64), budget=(256, 4096))
    st = O.build_centroids(wl)
    ref = O.decode_step(wl, st)                               # the selection does not depend on the scale
    want, want_lse = O.sparse_attention(wl, ref["sel_idx"], ref["sel_cnt"], sm_scale=scale)
    dw = _dev(wl)
    dw.layer.sm_scale = scale
    K = dw.sel_stride
    dw.sel_idx.copy_(torch.from_numpy(np.ascontiguousarray(ref["sel_idx"][:, :K])))
    dw.sel_cnt.copy_(torch.from_numpy(ref["sel_cnt"]))
    dw.sparse_decode()
    _check_out(dw, want, want_lse, f"sm_scale = {scale}, stand-alone")
    dw.build()
    dw.out.fill_(float("nan")); dw.lse.fill_(float("nan"))
    dw.decode_fused()
    _check_out(dw, want, want_lse, f"sm_scale = {scale}, fused")
    assert np.array_equal(dw.sel_idx.cpu().numpy(), ref["sel_idx"][:, :K])
    base = O.sparse_attention(wl, ref["sel_idx"], ref["sel_cnt"])[0]
    assert np.abs(base - want).max() > 1e-2                   # the scale does change the answer here


def test_non_finite_values_in_one_request_do_not_disturb_the_others_or_stall_anything():
    """Inputs are finite by contract; NaN and infinities must still not fault, hang or leak into other
    requests.  Request 0 gets a NaN and an infinity in its queries, keys and values: every call
    completes, no wait runs out, its lists are well formed (K_s ascending indices in range), and
    request 1 comes out exactly as the oracle has it."""
    from paper_2605_12110_amd import absb
    wl = synth.tiny_workload(seed=95, dtype=synth.F16, Bt=2, Hq=8, Hkv=2, P=16, seq_lens=(700, 500),
                             block_size=(8, 32), budget=(96, 128))
    nan, inf, ninf = np.uint16(0x7E00), np.uint16(0x7C00), np.uint16(0xFC00)
    wl.q[0, 1, 5] = nan
    wl.q[0, 6, 7] = inf
    pages0 = wl.page_table[0, :(700 + 15) // 16]
    wl.k_cache[pages0[3], 0, 2, 9] = nan
    wl.k_cache[pages0[5], 1, 1, 0] = inf
    wl.k_cache[pages0[7], 1, 4, 3] = ninf
    wl.v_cache[pages0[2], 0, 0, 1] = nan
    ref = O.decode_step(wl, O.build_centroids(wl))          # request 1 of it is untouched by all this
    dw = _dev(wl)
    K = dw.sel_stride
    for mode in (1, 2, 3):
        with _opts(dw, step_form=mode):
            dw.build()
            dw.sel_idx.fill_(-7); dw.sel_cnt.fill_(-7); dw.out.fill_(0); dw.lse.fill_(0)
            dw.decode_fused(); _sync()
        assert dw.status() == 0
        cnt, sel = dw.sel_cnt.cpu().numpy(), dw.sel_idx.cpu().numpy()
        assert np.array_equal(cnt, ref["sel_cnt"])                       # K_s does not depend on the data
        for s in range(4):
            b, h = divmod(s, 2)
            n = -(-int(wl.seq_lens[b]) // int(wl.block_size[h]))
            row = sel[s, :cnt[s]]
            assert np.all(row >= 0) and np.all(row < n) and np.all(np.diff(row) > 0) and np.all(sel[s, cnt[s]:] == -1)
        assert np.array_equal(sel[2:], ref["sel_idx"][2:, :K])           # request 1: bit-exact selection
        got = dw.out_f32().astype(np.float64)
        assert np.abs(got[1] - ref["out"][1]).max() <= TOL[wl.dtype]
        assert np.abs(dw.lse.cpu().numpy()[1].astype(np.float64) - ref["lse"][1]).max() <= LSE_TOL


# ------------------------------------------------------------------ randomised shapes
@pytest.mark.parametrize("seed", list(range(64)))
def test_random_shapes_modes_and_enqueue_forms(seed):
    """Seeded random small workloads over everything that shapes the path: batch, head counts and group
    size, page size, ragged lengths (down to one token), per-head block sizes on both sides of the page
    size, budgets from one block to beyond the context, dtype, block representation, who shares a
    selection, forced blocks.  Every stage against the oracle, the fused step in all its forms."""
    from paper_2605_12110_amd import absb
    rng = np.random.default_rng(1000 + seed)
    Bt = int(rng.integers(1, 5))
    Hkv = int(rng.integers(1, 4))
    G = int(rng.integers(1, 9))
    P = int(rng.choice([8, 16, 64, 128]))
    lens = [int(x) for x in rng.choice([1, 7, 64, 65, 300, 1023, 2048, 5000], size=Bt)]
    bs = [int(x) for x in rng.choice([8, 16, 32, 64, 128], size=Hkv)]
    budget = [int(x) for x in rng.choice([1, 8, 100, 512, 4096, 100000], size=Bt)]
    dtype = int(rng.choice([synth.F16, synth.BF16]))
    mode = int(rng.integers(0, 4))                 # 0 plain, 1 max-min pooling, 2 per query head, 3 group maximum
    wl = synth.tiny_workload(seed=2000 + seed, dtype=dtype, Bt=Bt, Hq=Hkv * G, Hkv=Hkv, P=P, seq_lens=lens,
                             block_size=bs, budget=budget)
    run_all_stages(wl, f"random {seed}: mode {mode}", block_repr=O.MINMAX if mode == 1 else O.MEAN,
                   per_query_head=mode == 2, group_max=mode == 3)


@pytest.mark.parametrize("seed", list(range(64)))
def test_random_shapes_with_few_distinct_keys_and_forced_blocks(seed):
    """As above on caches that hold 1, 2 or 17 distinct keys (one per page and head): whole runs of
    blocks score the same, so the selection lives on its tie paths and the softmax weights take few
    values; in the default mode also with forced first / last blocks through the fused step."""
    from paper_2605_12110_amd import absb
    rng = np.random.default_rng(3000 + seed)
    Bt = int(rng.integers(1, 5))
    Hkv = int(rng.integers(1, 4))
    G = int(rng.integers(1, 9))
    P = int(rng.choice([8, 16, 32, 64, 128, 256]))
    lens = [int(x) for x in rng.choice([1, 2, 9, 63, 65, 129, 300, 1024, 2049, 4097, 7000], size=Bt)]
    bs = [int(x) for x in rng.choice([8, 16, 32, 64, 128], size=Hkv)]
    budget = [int(x) for x in rng.choice([1, 7, 64, 500, 2048, 9000, 100000], size=Bt)]
    dtype = int(rng.choice([synth.F16, synth.BF16]))
    mode = int(rng.integers(0, 4))
    wl = synth.tiny_workload(seed=4000 + seed, dtype=dtype, Bt=Bt, Hq=Hkv * G, Hkv=Hkv, P=P, seq_lens=lens,
                             block_size=bs, budget=budget)
    m = int(rng.choice([1, 2, 17]))
    pal = synth.f32_to_bits(rng.standard_normal((m, wl.head_dim)).astype(np.float32), dtype)
    wl.k_cache[:] = pal[rng.integers(0, m, size=wl.k_cache.shape[:2])][:, :, None, :]
    run_all_stages(wl, f"few keys {seed}: mode {mode}, {m} keys", block_repr=O.MINMAX if mode == 1 else O.MEAN,
                   per_query_head=mode == 2, group_max=mode == 3)
    if mode == 0:
        sink, recent = int(rng.choice([0, 1, 9, 200, 5000])), int(rng.choice([0, 1, 65, 700, 5000]))
        st = O.build_centroids(wl)
        ref = O.decode_step(wl, st, sink_tokens=sink, recent_tokens=recent)
        dw = _dev(wl, sink_tokens=sink, recent_tokens=recent)
        dw.build()
        for form in (1, 2, 3):
            with _opts(dw, step_form=form):
                dw.sel_idx.fill_(-7); dw.sel_cnt.fill_(-7)
                dw.decode_fused()
                _check_out(dw, ref["out"], ref["lse"], f"forced sink={sink} recent={recent}, {FORMS[form]}")
            assert np.array_equal(dw.sel_cnt.cpu().numpy(), ref["sel_cnt"])
            assert np.array_equal(dw.sel_idx.cpu().numpy(), ref["sel_idx"][:, :dw.sel_stride])
            assert dw.status() == 0


# ------------------------------------------------------------------ per-query-head selection
@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
def test_per_query_head_selection_ragged_small_batch(dtype):
    wl = synth.tiny_workload(seed=5, dtype=dtype, Bt=3, Hq=8, Hkv=2, P=16, seq_lens=(37, 700, 1291),
                             block_size=(8, 32), budget=(64, 200, 96))
    run_all_stages(wl, f"per-query-head tiny dtype={dtype}", per_query_head=True)


@pytest.mark.parametrize("G", [1, 5, 8])
def test_per_query_head_selection_group_sizes(G):
    wl = synth.tiny_workload(seed=6, Bt=2, Hq=2 * G, Hkv=2, P=64, seq_lens=(1000, 2500), block_size=(128, 16),
                             budget=(256, 512))
    run_all_stages(wl, f"per-query-head G={G}", per_query_head=True)


def test_per_query_head_selection_config1_and_max_min_pooling():
    run_all_stages(synth.make_workload(1), "per-query-head config1", per_query_head=True)
    run_all_stages(synth.make_workload(1, context=2048, budget=256), "per-query-head config1/2K max-min",
                   block_repr=O.MINMAX, per_query_head=True)


def test_per_query_head_selection_config3_scaled():
    run_all_stages(synth.make_workload(3, context=32768, budget=2048), "per-query-head config3/32K",
                   per_query_head=True)


# ------------------------------------------------------------------ the group's maximum as the shared score
@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
def test_group_maximum_selection_ragged_small_batch(dtype):
    wl = synth.tiny_workload(seed=15, dtype=dtype, Bt=3, Hq=8, Hkv=2, P=16, seq_lens=(37, 700, 1291),
                             block_size=(8, 32), budget=(64, 200, 96))
    run_all_stages(wl, f"group-max tiny dtype={dtype}", group_max=True)


@pytest.mark.parametrize("G", [1, 3, 5, 8])
def test_group_maximum_selection_group_sizes(G):
    wl = synth.tiny_workload(seed=16, Bt=2, Hq=2 * G, Hkv=2, P=64, seq_lens=(1000, 2500), block_size=(128, 16),
                             budget=(256, 512))
    run_all_stages(wl, f"group-max G={G}", group_max=True)


def test_group_maximum_selection_config1_and_config3_scaled():
    run_all_stages(synth.make_workload(1), "group-max config1", group_max=True)
    run_all_stages(synth.make_workload(3, context=32768, budget=2048), "group-max config3/32K", group_max=True)


def test_group_maximum_selection_needs_the_offsets_and_mean_pooling():
    from paper_2605_12110_amd import absb
    wl = synth.tiny_workload(seed=17)
    dw = _dev(wl, selection=absb.SELECT_GROUP_MAX)
    dw.build()
    dw.batch.qmin = None
    with pytest.raises(absb.AbsbError) as e:
        dw.decode_fused()
    assert e.value.status == absb.ERR_NULL
    with pytest.raises(absb.AbsbError) as e:
        dw.score()
    assert e.value.status == absb.ERR_NULL
    with pytest.raises(absb.AbsbError) as e:
        _dev(wl, selection=absb.SELECT_GROUP_MAX, block_repr=absb.REPR_MINMAX)
    assert e.value.status == absb.ERR_UNSUPPORTED


# ------------------------------------------------------------------ the one-launch step beyond its default range
@pytest.mark.parametrize("context,sizes", [(131072, (8, 16)), (163840, (8, 8))])
def test_one_launch_step_on_segments_longer_than_the_default_allows(context, sizes):
    """By default a batch with a segment of more than 8192 blocks does not run as the pipelined
    one-launch step.  Forced into it, it must select the same blocks and give the same bits on every
    call: 16384 blocks (the longest register tile of the 256-thread selection) and 20480 blocks (keys
    re-read, no register tile: there the work list is the ascending list, and the bits are those of
    the per-stage form).  The unit form, the default beyond 16384 blocks, selects the same blocks."""
    import torch
    from paper_2605_12110_amd import absb
    wl = synth.make_workload(3, context=context, budget=4096, block_sizes=sizes)
    st = O.build_centroids(wl)
    ref = O.decode_step(wl, st)
    dw = _dev(wl)
    dw.build()
    assert absb.absb_step_form_used(dw.layer, dw.batch) == (absb.STEP_UNITS if context > 131072 else absb.STEP_PIPELINED)
    with _opts(dw, step_form=3):
        dw.decode_fused()
        _check_out(dw, ref["out"], ref["lse"], f"per stage, context {context}")
    assert np.array_equal(dw.sel_idx.cpu().numpy(), ref["sel_idx"][:, :dw.sel_stride])
    first = dw.out.clone() if context > 131072 else None
    for form in (1, 2, 0):
        with _opts(dw, step_form=form):
            for rep in range(2):                                     # twice: the counters must come back to zero
                dw.sel_idx.fill_(-7); dw.sel_cnt.fill_(-7); dw.out.fill_(float("nan")); dw.lse.fill_(float("nan"))
                dw.decode_fused()
                _check_out(dw, ref["out"], ref["lse"], f"form {form}, call {rep}, context {context}")
                if form == 1:
                    if first is None:
                        first = dw.out.clone()
                    assert torch.equal(dw.out, first), f"pipelined, call {rep}"
                assert np.array_equal(dw.sel_cnt.cpu().numpy(), ref["sel_cnt"])
                assert np.array_equal(dw.sel_idx.cpu().numpy(), ref["sel_idx"][:, :dw.sel_stride])
                assert dw.status() == 0
    head = dw.workspace[:dw.nseg * 6 * 256 + 256].view(torch.int32)
    assert int(head.abs().sum().item()) == 0, "the step left a counter, a flag or the status word set"


@pytest.mark.parametrize("form", [1, 2])
def test_one_launch_steps_back_to_back_and_on_two_streams(form):
    """The one-launch forms keep their hand-off counters in the workspace and leave them at zero: many
    steps enqueued without a synchronisation in between must each see clean counters, and two streams
    working on workspaces of their own must not disturb each other."""
    import torch
    from paper_2605_12110_amd import absb
    wls = [synth.make_workload(2, batch=2, context=8192, budget=1024, seed=s) for s in (41, 42)]
    refs = []
    for wl in wls:
        st = O.build_centroids(wl)
        refs.append(O.decode_step(wl, st))
    dws = [_dev(wl, opts=dict(step_form=form)) for wl in wls]
    for dw in dws:
        dw.build()
        assert absb.absb_step_form_used(dw.layer, dw.batch) == form
    _sync()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for st_ in streams:
        st_.wait_stream(torch.cuda.current_stream())
    for rep in range(25):                                   # interleaved enqueues, no synchronisation
        for dw, st_ in zip(dws, streams):
            with torch.cuda.stream(st_):
                dw.decode_fused(stream=st_)
    for st_ in streams:
        st_.synchronize()
    for dw, ref in zip(dws, refs):
        _check_out(dw, ref["out"], ref["lse"], "25 steps back to back, two streams")
        assert np.array_equal(dw.sel_cnt.cpu().numpy(), ref["sel_cnt"])
        assert np.array_equal(dw.sel_idx.cpu().numpy(), ref["sel_idx"][:, :dw.sel_stride])
        head = dw.workspace[:dw.nsel * 6 * 256 + 256].view(torch.int32)
        assert int(head.abs().sum().item()) == 0
        assert dw.status() == 0 and absb.absb_status_offset(dw.layer, dw.batch) == dw.nsel * 3 * 256


def test_one_workspace_serves_batches_of_different_shapes_when_cleared_in_between():
    """Requests join and leave: the same workspace runs a batch of three, of one, of five; its counters
    move with the number of segments, so absb_workspace_init runs whenever the shape changes."""
    from paper_2605_12110_amd import absb
    shapes = [((700, 65, 2049), (64, 2048, 100)), ((1500,), (256,)), ((9, 300, 4097, 64, 1023), (8, 64, 512, 4096, 100))]
    cases = []
    for i, (lens, budget) in enumerate(shapes):
        wl = synth.tiny_workload(seed=90 + i, dtype=synth.F16, Bt=len(lens), Hq=8, Hkv=2, P=16, seq_lens=lens,
                                 block_size=(8, 64), budget=budget)
        st = O.build_centroids(wl)
        cases.append((wl, O.decode_step(wl, st), _dev(wl)))
    shared = max((c[2].workspace for c in cases), key=lambda t: t.numel())
    for rnd in range(2):
        for wl, ref, dw in cases:
            dw.workspace = shared
            dw.build()                                   # leaves its scratch data where the next shape's counters sit
            dw.scribble(0xB7 + rnd)                      # = fill + absb_workspace_init for this shape
            for rep in range(4):                         # and no clearing between steps of one shape, whatever their form
                with _opts(dw, step_form=1 + rep % 2):
                    dw.sel_idx.fill_(-7); dw.out.fill_(float("nan"))
                    dw.decode_fused()
                    _check_out(dw, ref["out"], ref["lse"], f"shared workspace, batch of {wl.batch}, round {rnd}, step {rep}")
                assert np.array_equal(dw.sel_idx.cpu().numpy(), ref["sel_idx"][:, :dw.sel_stride])
                assert dw.status() == 0


@pytest.mark.parametrize("form", [1, 2])
def test_one_launch_step_gives_up_waiting_and_says_so_when_a_counter_was_not_cleared(form):
    """Work-groups of the one-launch forms wait for each other with a time limit.  Forced from the host:
    one segment's arrival counter starts at a value from which the count its work-groups wait for is
    never reached, so its list (pipelined form) or its threshold (unit form) never comes.  The launch
    must end by itself (about a quarter of a second per wait), set the status word, leave the other
    segments right, and write NaN into the stuck segment's output rows; after the counters
    are cleared again the step works."""
    import torch
    wl = synth.make_workload(1, context=4096, budget=256)
    ref = O.decode_step(wl, O.build_centroids(wl))
    dw = _dev(wl, opts=dict(step_form=form))
    dw.build()
    dw.decode_fused(); _sync()
    assert dw.status() == 0
    ctr = dw.workspace.view(torch.int32)
    stuck = 2
    ctr[(dw.nsel * 256) // 4 + stuck * 64] = 1000                # the arrival counters follow the attention tickets
    dw.sel_cnt.fill_(-7)
    t0 = time.time()
    dw.decode_fused(); _sync()
    took = time.time() - t0
    _say(f"    step with a stuck segment took {took:.2f} s")
    assert took < 5.0
    assert dw.status() == 1
    cnt = dw.sel_cnt.cpu().numpy()
    assert cnt[stuck] == -7                                       # nobody selected for the stuck segment
    others = [s for s in range(dw.nsel) if s != stuck]
    assert np.array_equal(cnt[others], ref["sel_cnt"][others])
    got = dw.out_f32().astype(np.float64)
    G = wl.group
    for s in others:
        assert np.abs(got[0, s * G:(s + 1) * G] - ref["out"][0, s * G:(s + 1) * G]).max() <= TOL[wl.dtype]
    assert np.isnan(got[0, stuck * G:(stuck + 1) * G]).all()
    dw.scribble(0x77)                                             # the contract: clear the counters, go on
    dw.decode_fused()
    _check_out(dw, ref["out"], ref["lse"], "after clearing the counters again")
    assert dw.status() == 0
    assert np.array_equal(dw.sel_idx.cpu().numpy(), ref["sel_idx"][:, :dw.sel_stride])


def test_one_launch_step_with_constant_keys_takes_the_tie_paths():
    """All keys of a head equal: every block of it scores the same, the threshold bin holds the whole
    segment (the crowded path of the selection) and the lowest indices must win, in both enqueue modes."""
    import torch
    from paper_2605_12110_amd import absb
    wl = synth.make_workload(1, context=16384, budget=1024, block_sizes=(8, 16))
    k = wl.k_cache.reshape(-1, wl.num_kv_heads, wl.page_size, wl.head_dim)
    k[:, 0] = k[0, 0, 0]                                         # KV head 0 (blocks of 16): one key everywhere
    k[:, 2] = k[0, 2, 0]                                         # KV head 2 (blocks of 8, 2048 of them): the same
    k[:, 1, :, 1:] = k[0, 1, 0, 1:]                              # KV head 1: keys differ in one channel only
    assert wl.block_size[0] == 16 and wl.block_size[2] == 8
    st = O.build_centroids(wl)
    ref = O.decode_step(wl, st)
    for h in (0, 2):
        assert np.array_equal(ref["sel_idx"][h, :ref["sel_cnt"][h]], np.arange(ref["sel_cnt"][h]))
    for mode in (1, 2, 3):
        dw = _dev(wl, opts=dict(step_form=mode))
        dw.build()
        dw.decode_fused()
        _check_out(dw, ref["out"], ref["lse"], f"constant keys, {FORMS[mode]}")
        assert np.array_equal(dw.sel_cnt.cpu().numpy(), ref["sel_cnt"])
        assert np.array_equal(dw.sel_idx.cpu().numpy(), ref["sel_idx"][:, :dw.sel_stride])
        assert dw.status() == 0


@pytest.mark.parametrize("distinct", [3, 40, 700])
def test_one_launch_step_on_long_segments_whose_scores_take_few_values(distinct):
    """Segments of 8192 and 16384 blocks (register tiles of 32 and 64 keys per thread in the pipelined
    form's selection) whose pages each hold one key out of a palette of 3, 40 or 700: the threshold bin holds
    from a few to thousands of equal scores, so the selection leaves its common path (members handed
    to the attention as they are found) for the ones that cut a long candidate list down, admit ties by
    index, or re-read a crowded bin, while other segments of the same launch stay on the common path.
    Every enqueue form must select the oracle's blocks, with and without the caller asking for the list."""
    wl = synth.make_workload(3, context=131072, budget=4096, block_sizes=(8, 16, 64))
    rng = np.random.default_rng(77 + distinct)
    k = wl.k_cache.reshape(-1, wl.num_kv_heads, wl.page_size, wl.head_dim)
    pal = synth.f32_to_bits(rng.standard_normal((distinct, wl.head_dim)).astype(np.float32), wl.dtype)
    for h in range(0, wl.num_kv_heads, 2):                        # every other KV head; the rest keep their keys
        k[:, h] = pal[rng.integers(0, distinct, size=k.shape[0])][:, None, :]   # one key per page: its blocks tie
    st = O.build_centroids(wl)
    ref = O.decode_step(wl, st)
    for mode in (1, 3):
        dw = _dev(wl, opts=dict(step_form=mode))
        dw.build()
        dw.sel_idx.fill_(-7); dw.sel_cnt.fill_(-7)
        dw.decode_fused()
        _check_out(dw, ref["out"], ref["lse"], f"{distinct} distinct keys, {FORMS[mode]}")
        assert np.array_equal(dw.sel_cnt.cpu().numpy(), ref["sel_cnt"])
        assert np.array_equal(dw.sel_idx.cpu().numpy(), ref["sel_idx"][:, :dw.sel_stride])
        first = dw.out.clone()
        dw.decode_fused(want_sel=False); _sync()
        import torch
        assert torch.equal(dw.out, first), "the list request changes the output"
        if mode == 1:
            assert dw.status() == 0


@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
def test_log_sum_exp_does_not_carry_the_rounding_of_the_weights(dtype):
    """Few distinct keys per head: every softmax weight of a kind rounds the same way when it is
    narrowed to the K/V type for the P V product (bf16: up to 2^-8 relative).  The output is
    normalised by the rounded weights (it stays a convex combination of value rows); the
    log-sum-exp must come from the weights before rounding and stay far inside its tolerance."""
    rng = np.random.default_rng(77)
    wl = synth.tiny_workload(seed=78, dtype=dtype, Bt=4, Hq=14, Hkv=2, P=8, seq_lens=(9, 65, 1000, 4097),
                             block_size=(16, 128), budget=(8, 2048, 100, 100000))
    pal = synth.f32_to_bits(rng.standard_normal((2, wl.head_dim)).astype(np.float32), dtype)
    pick = rng.integers(0, 2, size=wl.k_cache.shape[:2])
    wl.k_cache[:] = pal[pick][:, :, None, :]                     # two keys in all, one per page slab
    st = O.build_centroids(wl)
    ref = O.decode_step(wl, st)
    dw = _dev(wl)
    dw.build()
    dw.decode_fused()
    _check_out(dw, ref["out"], ref["lse"], "two distinct keys")
    lse = dw.lse.cpu().numpy().astype(np.float64)
    assert np.abs(lse - ref["lse"]).max() <= 2e-5


# ------------------------------------------------------------------ growing contexts (store maintenance)
def _view_at(wl, lens):
    import copy
    v = copy.copy(wl)
    v.seq_lens = np.asarray(lens, np.int32)
    return v


def _tight(dw, lens):
    """Rows in use of the capacity-layout code array, in the tight layout of the given lengths."""
    codes = dw.codes.cpu().numpy()
    off = dw.plan.cent_off
    rows = []
    Hkv = dw.wl.num_kv_heads
    for s in range(dw.nseg):
        b, h = divmod(s, Hkv)
        n = -(-int(lens[b]) // int(dw.block_size[h]))
        rows.append(codes[off[s]:off[s] + n])
    return np.concatenate(rows)


@pytest.mark.parametrize("repr_,dtype", [(O.MEAN, synth.F16), (O.MEAN, synth.BF16), (O.MINMAX, synth.F16)])
def test_appending_tokens_keeps_the_store_and_the_step_in_parity(repr_, dtype):
    """Contexts grow token by token inside a layout sized for the final lengths: tail state and code
    rows bit-exact against the oracle after every token, and the fused step on the grown store
    (selection bit-exact, outputs within tolerance) at a few points on the way."""
    full = synth.tiny_workload(seed=71, dtype=dtype, Bt=3, Hq=8, Hkv=2, P=16, seq_lens=(150, 97, 1300),
                               block_size=(8, 32), budget=(32, 24, 200))
    grow = 45
    start = full.seq_lens - grow
    view = _view_at(full, start)
    dw = _dev(view, block_repr=repr_, cap_lens=full.seq_lens)
    assert dw.plan.cent_off[-1] == O.offsets(full)[-1]                # laid out for the final lengths
    _say(f"[case append repr={repr_} dtype={dtype}] start={start.tolist()} -> {full.seq_lens.tolist()}")
    dw.build(); dw.tail_init(); _sync()
    store = O.build_centroids(view, repr_)
    tail = O.tail_state(view, repr_)
    assert np.array_equal(_tight(dw, start), store.codes) and np.array_equal(dw.qscale.cpu().numpy(), store.qscale)
    assert np.array_equal(dw.tail.cpu().numpy(), tail)
    clamped = np.zeros(dw.nseg, np.int32)              # values of completed blocks outside the frozen ranges
    for step in range(1, grow + 1):
        lens = start + step
        view = _view_at(full, lens)
        dw.wl = view
        dw.set_lens(lens)
        dw.append_token()
        store, _ = O.append_token(view, store, tail, clamped)
        _sync()
        assert np.array_equal(dw.tail.cpu().numpy(), tail), f"tail state after {step} tokens"
        assert np.array_equal(_tight(dw, lens), store.codes), f"code rows after {step} tokens"
        assert np.array_equal(dw.clamped.cpu().numpy(), clamped), f"re-ranging counters after {step} tokens"
        if step in (1, 7, 8, 9, 32, grow):
            ref = O.decode_step(view, store)
            dw.sel_idx.fill_(-7); dw.sel_cnt.fill_(-7); dw.out.fill_(float("nan")); dw.lse.fill_(float("nan"))
            dw.decode_fused()
            _check_out(dw, ref["out"], ref["lse"], f"fused step after {step} appended tokens")
            K = dw.sel_stride
            assert np.array_equal(dw.sel_cnt.cpu().numpy(), ref["sel_cnt"])
            got = dw.sel_idx.cpu().numpy()
            kk = min(K, ref["sel_idx"].shape[1])
            assert np.array_equal(got[:, :kk], ref["sel_idx"][:, :kk]) and np.all(got[:, kk:] == -1)
    assert clamped.sum() > 0                           # the counters were exercised


def test_lists_widen_with_the_context_when_the_budget_exceeds_it():
    """A budget beyond the context selects every block, so K_s and the list width that absb_plan
    reports grow with the lengths: the fused step writes [segments][that width] for the lengths
    of the call, inside a buffer sized for the longest contexts."""
    full = synth.tiny_workload(seed=73, dtype=synth.F16, Bt=3, Hq=15, Hkv=3, P=8, seq_lens=(3020, 85, 148),
                               block_size=(64, 16, 128), budget=(8, 4096, 8))
    start = full.seq_lens - 20
    view = _view_at(full, start)
    dw = _dev(view, cap_lens=full.seq_lens)
    dw.build(); dw.tail_init(); _sync()
    store = O.build_centroids(view)
    tail = O.tail_state(view)
    widths = set()
    for step in range(1, 21):
        lens = start + step
        view = _view_at(full, lens)
        dw.wl = view
        dw.set_lens(lens)
        dw.append_token()
        store, _ = O.append_token(view, store, tail)
        ref = O.decode_step(view, store)
        dw.sel_idx.fill_(-7); dw.sel_cnt.fill_(-7)
        dw.decode_fused()
        _check_out(dw, ref["out"], ref["lse"], f"after {step} tokens")
        K = dw.sel_stride
        widths.add(K)
        assert K == int(ref["sel_cnt"].max())
        assert np.array_equal(dw.sel_cnt.cpu().numpy(), ref["sel_cnt"])
        assert np.array_equal(dw.sel_idx.cpu().numpy(), ref["sel_idx"][:, :K])
    assert len(widths) > 1


def test_one_request_of_a_batch_is_re_ranged_in_place():
    """Re-ranging one request without touching the others: a batch of one (that request's lengths,
    page-table row and capacity) whose code, scale and offset pointers point into the batch's arrays
    at the request's first segment.  Its rows and ranges become those of a fresh build at the new
    length; every other request's stay bit for bit; the step on the mixed store matches the oracle."""
    import torch
    from paper_2605_12110_amd import absb
    full = synth.tiny_workload(seed=74, dtype=synth.F16, Bt=3, Hq=8, Hkv=2, P=16, seq_lens=(400, 333, 900),
                               block_size=(8, 32), budget=(64, 64, 128))
    start = full.seq_lens - 60
    view = _view_at(full, start)
    dw = _dev(view, cap_lens=full.seq_lens)
    dw.build(); dw.tail_init(); _sync()
    store = O.build_centroids(view)
    tail = O.tail_state(view)
    for step in range(1, 61):                                # grow all three requests under frozen ranges
        lens = start + step
        view = _view_at(full, lens)
        dw.wl = view
        dw.set_lens(lens)
        dw.append_token()
        store, _ = O.append_token(view, store, tail)
    _sync()
    before_codes, before_scale, before_min = dw.codes.cpu().numpy(), dw.qscale.cpu().numpy(), dw.qmin.cpu().numpy()
    assert np.array_equal(_tight(dw, lens), store.codes)

    b, Hkv = 1, full.num_kv_heads
    one_lens = full.seq_lens[b:b + 1].copy()
    sub = absb.Batch(seq_lens_host=one_lens, budget_host=full.budget[b:b + 1].copy(), seq_lens=dw.seq_lens[b:b + 1],
                     page_table=dw.page_table[b:b + 1], budget=dw.budget[b:b + 1], pt_stride=dw.page_table.shape[1])
    sub.cap_lens_host = one_lens
    sub_plan = absb.absb_plan(dw.layer, sub)
    sub_off = sub_plan.cent_off
    base = int(dw.plan.cent_off[b * Hkv])
    assert np.array_equal(sub_off, dw.plan.cent_off[b * Hkv:(b + 1) * Hkv + 1] - base)   # same layout, shifted
    sub.cent_off = torch.from_numpy(sub_off).to(dw.device)
    # a workspace of its own: the counters at the start of a workspace belong to one batch shape
    ws = torch.empty((sub_plan.workspace_bytes,), dtype=torch.uint8, device=dw.device)
    absb.absb_build_centroids(dw.layer, sub, dw.k_cache, dw.codes[base:], dw.qscale[b * Hkv:], dw.qmin[b * Hkv:], ws)
    _sync()
    fresh = O.build_centroids(view)                          # every request rebuilt: request b must match this one
    codes, scale, mn = dw.codes.cpu().numpy(), dw.qscale.cpu().numpy(), dw.qmin.cpu().numpy()
    off = dw.plan.cent_off
    for s in range(dw.nseg):
        n = -(-int(lens[s // Hkv]) // int(dw.block_size[s % Hkv]))
        rows = slice(int(off[s]), int(off[s]) + n)
        if s // Hkv == b:
            assert np.array_equal(codes[rows], fresh.codes[fresh.off[s]:fresh.off[s + 1]])
            assert np.array_equal(scale[s], fresh.qscale[s]) and np.array_equal(mn[s], fresh.qmin[s])
        else:
            assert np.array_equal(codes[rows], before_codes[rows])
            assert np.array_equal(scale[s], before_scale[s]) and np.array_equal(mn[s], before_min[s])
    assert not np.array_equal(scale[b * Hkv], before_scale[b * Hkv])      # the ranges did move
    # the step on the mixed store: the oracle's store with request b's segments replaced
    import copy
    mixed = copy.copy(store)
    mixed.codes, mixed.qscale, mixed.qmin = store.codes.copy(), store.qscale.copy(), store.qmin.copy()
    for s in range(b * Hkv, (b + 1) * Hkv):
        mixed.codes[mixed.off[s]:mixed.off[s + 1]] = fresh.codes[fresh.off[s]:fresh.off[s + 1]]
        mixed.qscale[s], mixed.qmin[s] = fresh.qscale[s], fresh.qmin[s]
    ref = O.decode_step(view, mixed)
    dw.decode_fused()
    _check_out(dw, ref["out"], ref["lse"], "step after re-ranging one request")
    assert np.array_equal(dw.sel_idx.cpu().numpy(), ref["sel_idx"][:, :dw.sel_stride])


def test_stages_ignore_the_unused_rows_of_a_layout_sized_for_longer_contexts():
    """A store laid out for longer contexts than the current ones: build, score, selection and the
    step give the same results as the tight layout (the unused rows hold garbage)."""
    full = synth.tiny_workload(seed=72, dtype=synth.F16, Bt=2, Hq=8, Hkv=4, P=16, seq_lens=(999, 2500),
                               block_size=(128, 8, 64, 16), budget=(300, 520))
    lens = np.array([700, 1801], np.int32)
    view = _view_at(full, lens)
    st = O.build_centroids(view)
    ref = O.decode_step(view, st)
    dw = _dev(view, cap_lens=full.seq_lens)
    dw.codes.fill_(0xEE); dw.scores.fill_(2 ** 31 - 1)               # garbage in every row, used or not
    dw.build(); _sync()
    assert np.array_equal(_tight(dw, lens), st.codes)
    assert np.array_equal(dw.qscale.cpu().numpy(), st.qscale) and np.array_equal(dw.qmin.cpu().numpy(), st.qmin)
    dw.decode_fused()
    _check_out(dw, ref["out"], ref["lse"], "capacity layout")
    kk = min(dw.sel_stride, ref["sel_idx"].shape[1])
    assert np.array_equal(dw.sel_cnt.cpu().numpy(), ref["sel_cnt"])
    assert np.array_equal(dw.sel_idx.cpu().numpy()[:, :kk], ref["sel_idx"][:, :kk])


# ------------------------------------------------------------------ graph capture
def test_fused_step_replays_from_a_captured_graph():
    """The fused step enqueues kernels only (no memsets, no allocation, no synchronisation), so it can
    be captured once and replayed: every replay, with eager work and synchronisations in between,
    must give the eager step's bits, also after the query has changed in place."""
    import torch
    wl = synth.make_workload(1, context=8192, budget=1024)
    st = O.build_centroids(wl)
    ref = O.decode_step(wl, st)
    dw = _dev(wl)
    dw.build()
    dw.decode_fused(); _sync()
    eager = dw.out.clone(); eager_sel = dw.sel_idx.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        dw.decode_fused()                                   # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            dw.decode_fused()
    torch.cuda.current_stream().wait_stream(side)
    _sync()
    for rep in range(4):
        dw.out.fill_(float("nan")); dw.sel_idx.fill_(-7)
        dw.scribble(0x11 * (rep + 1))                       # eager work between the replays
        _sync()
        graph.replay()
        _sync()
        assert torch.equal(dw.out, eager) and torch.equal(dw.sel_idx, eager_sel), f"replay {rep}"
    _check_out(dw, ref["out"], ref["lse"], "graph replay")
    # new inputs in place (the next decode step's query): the replay follows them
    wl2 = synth.make_workload(1, context=8192, budget=1024, seed=999)
    dw.q.copy_(torch.from_numpy(wl2.q.view(np.int16)).view(dw.torch_dtype).to(dw.q.device))
    wl.q = wl2.q
    ref2 = O.decode_step(wl, st)
    graph.replay()
    _check_out(dw, ref2["out"], ref2["lse"], "graph replay, new query")
    assert np.array_equal(dw.sel_idx.cpu().numpy(), ref2["sel_idx"][:, :dw.sel_stride])
