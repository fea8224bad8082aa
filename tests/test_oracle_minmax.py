"""Pins for the oracle's max-min block representation (no GPU).

The representation is the max-min pooling named in the footnote of Sec. 2.2 (the estimator of
the baseline in Sec. 4.1): per block the channel-wise maxima and minima of its keys, scored by
sum_c max(q_c * max_c, q_c * min_c), an upper bound of q . k over the block.  Pinned against
numpy extrema, the bound property itself, an fp64 evaluation of the max formula on the
dequantized codes, hand-built integer cases, and the reductions to the mean representation's
arithmetic that the two share (quantizer, fixed-point image).
"""
import numpy as np
import pytest

from oracle import oracle as O
from paper_2605_12110_amd import synth


def _unpack(codes):
    return np.stack([codes & 15, codes >> 4], axis=-1).reshape(codes.shape[0], -1).astype(np.int64)


def _pack(cu):
    cu = np.asarray(cu, dtype=np.uint8)
    return np.ascontiguousarray((cu[:, 0::2] | (cu[:, 1::2] << 4)).astype(np.uint8))


def _store(cu_max, cu_min, scale_max, scale_min, off):
    nseg = len(off) - 1
    codes = np.ascontiguousarray(np.concatenate([_pack(cu_max), _pack(cu_min)], axis=1))
    qs = np.concatenate([np.broadcast_to(np.asarray(scale_max, np.float32), (nseg, 128)),
                         np.broadcast_to(np.asarray(scale_min, np.float32), (nseg, 128))], axis=1).copy()
    return O.CentroidStore(np.asarray(off, np.int64), None, qs, np.zeros_like(qs), np.zeros_like(qs), codes, O.MINMAX)


def _wl_with_q(qf32, Hkv, dtype=synth.F16):
    Bt, Hq, _ = qf32.shape
    wl = synth.tiny_workload(dtype=dtype, Bt=Bt, Hq=Hq, Hkv=Hkv, P=16, seq_lens=(64,) * Bt,
                             block_size=(8,) * Hkv, budget=(8,) * Bt)
    wl.q = synth.f32_to_bits(qf32, dtype)
    return wl


# ------------------------------------------------------------------ pooling
@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
def test_pool_is_the_channelwise_extrema_of_each_blocks_keys(dtype):
    wl = synth.tiny_workload(seed=5, dtype=dtype, Bt=2, Hq=4, Hkv=2, P=16, seq_lens=(203, 64),
                             block_size=(8, 32), budget=(64, 64))
    off = O.offsets(wl)
    rep = O.minmax_pool(wl, off)
    assert rep.shape == (int(off[-1]), 256)
    for s in range(4):
        b, h = divmod(s, 2)
        K = wl.key_rows(b, h)
        B = int(wl.block_size[h])
        for j in range(int(off[s + 1] - off[s])):
            blk = K[j * B:(j + 1) * B]                      # the last block of request 0 is partial
            assert np.array_equal(rep[off[s] + j, :128], blk.max(axis=0))
            assert np.array_equal(rep[off[s] + j, 128:], blk.min(axis=0))


def test_pool_is_invariant_under_page_permutation_and_exact_for_constant_blocks():
    a = synth.tiny_workload(seed=9, Bt=1, Hq=2, Hkv=1, P=16, seq_lens=(100,), block_size=(32,), budget=(32,),
                            shuffle_pages=False)
    b = synth.tiny_workload(seed=9, Bt=1, Hq=2, Hkv=1, P=16, seq_lens=(100,), block_size=(32,), budget=(32,),
                            shuffle_pages=True)
    # same logical keys behind different page tables
    for t in range(100):
        b.k_cache[b.page_table[0, t // 16], 0, t % 16] = a.k_cache[a.page_table[0, t // 16], 0, t % 16]
    ra, rb = O.minmax_pool(a, O.offsets(a)), O.minmax_pool(b, O.offsets(b))
    assert np.array_equal(ra, rb)
    # a block of identical keys: maxima == minima == the key
    a.k_cache[a.page_table[0, 2], 0, :] = a.k_cache[a.page_table[0, 2], 0, 0]
    a.k_cache[a.page_table[0, 3], 0, :] = a.k_cache[a.page_table[0, 2], 0, 0]
    r = O.minmax_pool(a, O.offsets(a))
    key = synth.bits_to_f32(a.k_cache[a.page_table[0, 2], 0, 0], a.dtype)
    assert np.array_equal(r[1, :128], key) and np.array_equal(r[1, 128:], key)


def test_unquantized_score_bounds_every_tokens_logit_from_above():
    # the reason for the representation: sum_c max(q_c M_c, q_c m_c) >= q . k_t for every token of the block
    wl = synth.make_workload(1, context=1024)
    off = O.offsets(wl)
    rep = O.minmax_pool(wl, off).astype(np.float64)
    q = synth.bits_to_f32(wl.q, wl.dtype).astype(np.float64)
    G = wl.group
    for s in range(wl.num_kv_heads):
        K = wl.key_rows(0, s).astype(np.float64)
        B = int(wl.block_size[s])
        for g in range(G):
            qv = q[0, s * G + g]
            M, m = rep[off[s]:off[s + 1], :128], rep[off[s]:off[s + 1], 128:]
            ub = np.maximum(qv * M, qv * m).sum(axis=1)
            logits = (K @ qv).reshape(-1, B)
            assert np.all(ub[:, None] >= logits - 1e-9)
            assert np.all(ub - logits.max(axis=1) >= -1e-9)


# ------------------------------------------------------------------ store
def test_store_quantizes_maxima_and_minima_with_their_own_channel_ranges():
    wl = synth.make_workload(1, context=1024)
    st = O.build_centroids(wl, O.MINMAX)
    assert st.codes.shape == (int(st.off[-1]), 128) and st.qscale.shape == (wl.num_kv_heads, 256)
    for s in range(wl.num_kv_heads):
        blk = st.cent[st.off[s]:st.off[s + 1]].astype(np.float64)
        lo, hi = blk.min(axis=0), blk.max(axis=0)
        assert np.array_equal(st.qmin[s].astype(np.float64), lo)
        assert np.allclose(st.qscale[s], (hi - lo) / 15.0, rtol=1e-6, atol=0)
        cu = _unpack(st.codes[st.off[s]:st.off[s + 1]])
        assert cu.shape[1] == 256 and cu.min() >= 0 and cu.max() <= 15
        # every channel of both halves reaches both ends of its own range
        assert np.all(cu.min(axis=0) == 0) and np.all(cu.max(axis=0) == 15)
        deq = cu * st.qscale[s].astype(np.float64) + lo
        assert np.all(np.abs(deq - blk) <= st.qscale[s].astype(np.float64) / 2 * (1 + 1e-5) + 1e-12)


# ------------------------------------------------------------------ score
def test_score_hand_case_sign_split_weights():
    # one KV head, G = 2.  Channel 0: q = (+0.5, +0.5) -> P = 1,    Q = 0
    #                     channel 1: q = (+0.5, -0.25) -> P = 0.5, Q = -0.25
    #                     channel 2: q = (-0.5, -0.5) -> P = 0,    Q = -1
    # scales 1: A = 1, exponent -14, weights on maxima [16384, 8192, 0], on minima [0, -4096, -16384]
    q = np.zeros((1, 2, 128), np.float32)
    q[0, 0, :3] = [0.5, 0.5, -0.5]
    q[0, 1, :3] = [0.5, -0.25, -0.5]
    wl = _wl_with_q(q, Hkv=1)
    rng = np.random.default_rng(0)
    cM, cm = rng.integers(0, 16, size=(8, 128)), rng.integers(0, 16, size=(8, 128))
    st = _store(cM, cm, 1.0, 1.0, [0, 8])
    scores, ex, wq = O.score(wl, st, want_weights=True)
    assert ex[0] == -14 and wq.shape == (1, 256)
    assert list(wq[0, :4]) == [16384, 8192, 0, 0] and list(wq[0, 128:132]) == [0, -4096, -16384, 0]
    assert not wq[0, 4:128].any() and not wq[0, 132:].any()
    want = [16384 * int(a[0]) + 8192 * int(a[1]) - 4096 * int(b[1]) - 16384 * int(b[2]) for a, b in zip(cM, cm)]
    assert list(scores) == want


def test_score_is_the_integer_dot_of_the_reported_weights_and_tops_out_in_range():
    rng = np.random.default_rng(1)
    q = rng.standard_normal((2, 10, 128)).astype(np.float32)            # G = 5
    wl = _wl_with_q(q, Hkv=2, dtype=synth.BF16)
    cM, cm = rng.integers(0, 16, size=(40, 128)), rng.integers(0, 16, size=(40, 128))
    st = _store(cM, cm, 1.0, 1.0, [0, 10, 20, 30, 40])
    st.qscale[:] = (np.abs(rng.standard_normal((4, 256))) + 0.01).astype(np.float32)
    scores, ex, wq = O.score(wl, st, want_weights=True)
    top = np.abs(wq).max(axis=1)
    assert np.all(top >= 16384) and np.all(top <= 32768)
    assert np.all(wq[:, :128] >= 0) and np.all(wq[:, 128:] <= 0)        # maxima meet positive, minima negative parts
    cu = _unpack(st.codes)
    want = np.concatenate([cu[st.off[s]:st.off[s + 1]] @ wq[s].astype(np.int64) for s in range(4)])
    assert np.array_equal(scores.astype(np.int64), want)


@pytest.mark.parametrize("cfg", [1, 2, 4])
def test_score_tracks_the_fp64_max_formula_on_the_dequantized_extrema(cfg):
    """2^e S_j + const = sum_g sum_c [q_gc > 0 ? q_gc M^_jc : q_gc m^_jc] within the weight-rounding bound,
    and that equals the literal sum_g sum_c max(q_gc M^_jc, q_gc m^_jc) for every block whose dequantized
    maxima are not below its dequantized minima; where they cross, the literal max can only be larger."""
    wl = synth.make_workload(cfg, context=2048, batch=2)
    st = O.build_centroids(wl, O.MINMAX)
    scores, ex = O.score(wl, st)
    q = synth.bits_to_f32(wl.q, wl.dtype).astype(np.float64)
    G = wl.group
    seen_clean = 0
    for s in range(len(st.off) - 1):
        b, h = divmod(s, wl.num_kv_heads)
        lo, hi = st.off[s], st.off[s + 1]
        cu = _unpack(st.codes[lo:hi]).astype(np.float64)
        deq = cu * st.qscale[s].astype(np.float64) + st.qmin[s].astype(np.float64)
        M, m = deq[:, :128], deq[:, 128:]
        qs = q[b, h * G:(h + 1) * G]
        literal = sum(np.maximum(qv * M, qv * m).sum(axis=1) for qv in qs)
        matched = sum((np.where(qv > 0, qv, 0) * M + np.where(qv < 0, qv, 0) * m).sum(axis=1) for qv in qs)
        P, Q = np.where(qs > 0, qs, 0).sum(axis=0), np.where(qs < 0, qs, 0).sum(axis=0)
        const = P @ st.qmin[s, :128].astype(np.float64) + Q @ st.qmin[s, 128:].astype(np.float64)
        est = np.ldexp(scores[lo:hi].astype(np.float64), int(ex[s])) + const
        bound = 256 * 15 * 2.0 ** (int(ex[s]) - 1) * 1.05 + 1e-3 * np.abs(matched).max() * 2.0 ** -10
        assert np.abs(est - matched).max() <= bound
        assert np.all(literal >= matched - 1e-9)
        clean = np.all(M >= m, axis=1)
        seen_clean += int(clean.sum())
        assert np.allclose(literal[clean], matched[clean], rtol=1e-12, atol=1e-9)
    assert seen_clean > 0


def test_score_reduces_to_a_plain_dot_when_maxima_equal_minima():
    # blocks of identical keys: M = m = k, so the bound is q . k itself and the ranking that of the exact logits
    wl = synth.tiny_workload(seed=3, Bt=1, Hq=1, Hkv=1, P=16, seq_lens=(256,), block_size=(8,), budget=(8,))
    for j in range(32):
        pg, sl = wl.page_table[0, (8 * j) // 16], (8 * j) % 16
        wl.k_cache[pg, 0, sl:sl + 8] = wl.k_cache[pg, 0, sl]
    st = O.build_centroids(wl, O.MINMAX)
    assert np.array_equal(st.cent[:, :128], st.cent[:, 128:])
    assert np.array_equal(st.codes[:, :64], st.codes[:, 64:]) and np.array_equal(st.qscale[:, :128], st.qscale[:, 128:])
    scores, ex = O.score(wl, st)
    qv = synth.bits_to_f32(wl.q, wl.dtype).astype(np.float64)[0, 0]
    cu = _unpack(st.codes[:, :64]).astype(np.float64)
    deq_dot = (cu * st.qscale[0, :128].astype(np.float64)) @ qv          # q . (k^ - min), the ranking term
    est = np.ldexp(scores.astype(np.float64), int(ex[0]))
    assert np.abs(est - deq_dot).max() <= 256 * 15 * 2.0 ** (int(ex[0]) - 1) * 1.05


def test_score_degenerate_inputs():
    wl = _wl_with_q(np.zeros((1, 2, 128), np.float32), Hkv=1)
    st = _store(np.full((5, 128), 7), np.full((5, 128), 3), 1.0, 1.0, [0, 5])
    scores, ex = O.score(wl, st)
    assert not scores.any() and ex[0] == 0
    q = np.ones((1, 2, 128), np.float32)                                 # all positive: only the maxima count
    scores, _ = O.score(_wl_with_q(q, 1), st)
    st2 = _store(np.full((5, 128), 7), np.full((5, 128), 12), 1.0, 1.0, [0, 5])
    scores2, _ = O.score(_wl_with_q(q, 1), st2)
    assert np.array_equal(scores, scores2) and len(set(scores.tolist())) == 1
    scores3, _ = O.score(_wl_with_q(-q, 1), st2)                         # all negative: only the minima count
    scores4, _ = O.score(_wl_with_q(-q, 1), st)
    assert scores3[0] < scores4[0] < 0


def test_step_with_the_max_min_store_finds_the_planted_tokens():
    wl = synth.make_workload(1, context=2048)
    st = O.build_centroids(wl, O.MINMAX)
    r = O.decode_step(wl, st)
    assert O.planted_recall(wl, r["sel_idx"], r["sel_cnt"]) >= 0.8
    tokens = (r["sel_cnt"].reshape(1, -1) * wl.block_size).ravel()
    assert np.all(tokens == np.minimum(wl.budget[0], wl.seq_lens[0]))
