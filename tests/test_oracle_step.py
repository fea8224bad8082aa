"""Pins for the oracle's per-step path: fixed-point score, Top-K, sparse attention (no GPU).

Pinned against: independent integer arithmetic on hand-built cases, an fp64 evaluation
of the paper's importance score r_j = q . c_j^T (Sec. 2.2) within its derived error bound,
numpy lexsort and exhaustive tiny cases for the selection, the K_h = ceil(T/B_h) rule
(Sec. 3.4, kernel 2), and an independent numpy evaluation of Eq. (1) for attention.
"""
import itertools

import numpy as np
import pytest

from oracle import oracle as O
from paper_2605_12110_amd import synth


def _unpack(codes):
    return np.stack([codes & 15, codes >> 4], axis=-1).reshape(codes.shape[0], -1).astype(np.int64)


def _store_from(codes_unpacked, qscale, off):
    cu = np.asarray(codes_unpacked, dtype=np.uint8)
    packed = np.ascontiguousarray((cu[:, 0::2] | (cu[:, 1::2] << 4)).astype(np.uint8))
    nseg = len(off) - 1
    qs = np.broadcast_to(np.asarray(qscale, np.float32), (nseg, cu.shape[1])).copy()
    return O.CentroidStore(np.asarray(off, np.int64), None, qs, np.zeros_like(qs), np.zeros_like(qs), packed)


def _wl_with_q(qf32, Hkv, dtype=synth.F16, L=64):
    Bt, Hq, _ = qf32.shape
    wl = synth.tiny_workload(dtype=dtype, Bt=Bt, Hq=Hq, Hkv=Hkv, P=16, seq_lens=(L,) * Bt,
                             block_size=(8,) * Hkv, budget=(8,) * Bt)
    wl.q = synth.f32_to_bits(qf32, dtype)
    return wl


# ------------------------------------------------------------------ O4 score
def test_score_hand_case_powers_of_two():
    # one KV head, G = 2: u = q0 + q1 = [1, 0.5, -0.25, 0, ...]; scale 1 => A = 1, exponent -14,
    # integer weights [16384, 8192, -4096, 0...]; scores are plain integer dot products.
    q = np.zeros((1, 2, 128), np.float32)
    q[0, 0, :3] = [0.75, 0.25, -0.125]
    q[0, 1, :3] = [0.25, 0.25, -0.125]
    wl = _wl_with_q(q, Hkv=1)
    rng = np.random.default_rng(0)
    cu = rng.integers(0, 16, size=(8, 128))
    st = _store_from(cu, 1.0, [0, 8])
    scores, ex, wq = O.score(wl, st, want_weights=True)
    assert ex[0] == -14
    assert list(wq[0, :4]) == [16384, 8192, -4096, 0] and not wq[0, 4:].any()
    want = [16384 * int(c[0]) + 8192 * int(c[1]) - 4096 * int(c[2]) for c in cu]
    assert list(scores) == want


def test_score_weight_image_tops_out_in_2e14_2e15():
    rng = np.random.default_rng(1)
    q = rng.standard_normal((2, 8, 128)).astype(np.float32)
    wl = _wl_with_q(q, Hkv=2)
    cu = rng.integers(0, 16, size=(40, 128))
    qs = np.abs(rng.standard_normal((4, 128))).astype(np.float32) + 0.01
    st = _store_from(cu, 1.0, [0, 10, 20, 30, 40])
    st.qscale[:] = qs
    scores, ex, wq = O.score(wl, st, want_weights=True)
    top = np.abs(wq).max(axis=1)
    assert np.all(top >= 16384) and np.all(top <= 32768)
    # independent integer dot with the reported weights
    want = np.concatenate([_unpack(st.codes)[st.off[s]:st.off[s + 1]] @ wq[s].astype(np.int64) for s in range(4)])
    assert np.array_equal(scores.astype(np.int64), want)


def test_score_is_invariant_under_channel_permutation():
    # integer accumulation: any channel order must give identical scores (permute in byte pairs
    # and within pairs consistently for q, scale and codes)
    rng = np.random.default_rng(2)
    q = rng.standard_normal((1, 4, 128)).astype(np.float32)
    cu = rng.integers(0, 16, size=(33, 128))
    qs = (np.abs(rng.standard_normal((1, 128))) + 0.1).astype(np.float32)
    perm = rng.permutation(128)
    a = _store_from(cu, 1.0, [0, 33]); a.qscale[:] = qs
    b = _store_from(cu[:, perm], 1.0, [0, 33]); b.qscale[:] = qs[:, perm]
    sa, ea = O.score(_wl_with_q(q, 1), a)
    sb, eb = O.score(_wl_with_q(q[:, :, perm], 1), b)
    assert np.array_equal(sa, sb) and np.array_equal(ea, eb)


@pytest.mark.parametrize("cfg,dtype_G", [(1, "f16 G4"), (2, "bf16 G4"), (4, "bf16 G5")])
def test_score_tracks_the_dequantized_dot_product_within_bound(cfg, dtype_G):
    # |2^e S_j + sum_c u_c min_c - sum_g q_g . c^_j| <= d * 15 * 2^(e-1) (weight rounding), all in fp64
    wl = synth.make_workload(cfg, context=2048, batch=2)
    st = O.build_centroids(wl)
    scores, ex = O.score(wl, st)
    deq = O.dequantize(st.off, st.codes, st.qscale, st.qmin).astype(np.float64)
    q = synth.bits_to_f32(wl.q, wl.dtype).astype(np.float64)
    G = wl.group
    for s in range(len(st.off) - 1):
        b, h = divmod(s, wl.num_kv_heads)
        lo, hi = st.off[s], st.off[s + 1]
        r = sum(deq[lo:hi] @ q[b, h * G + g] for g in range(G))          # the paper's score, summed over the group
        u = q[b, h * G:(h + 1) * G].sum(axis=0)
        est = np.ldexp(scores[lo:hi].astype(np.float64), int(ex[s])) + u @ st.qmin[s].astype(np.float64)
        bound = 128 * 15 * 2.0 ** (int(ex[s]) - 1) * 1.05 + 1e-3 * np.abs(r).max() * 2.0 ** -10
        assert np.abs(est - r).max() <= bound


def test_score_one_hot_query_ranks_by_that_channels_codes():
    q = np.zeros((1, 1, 128), np.float32)
    q[0, 0, 77] = 3.0
    wl = _wl_with_q(q, Hkv=1)
    rng = np.random.default_rng(3)
    cu = rng.integers(0, 16, size=(50, 128))
    st = _store_from(cu, 0.37, [0, 50])
    scores, ex = O.score(wl, st)
    assert np.array_equal(np.argsort(scores, kind="stable"), np.argsort(cu[:, 77], kind="stable"))
    q[0, 0, 77] = -3.0                               # negative weight reverses the order
    scores, _ = O.score(_wl_with_q(q, 1), st)
    assert np.array_equal(np.argsort(-scores, kind="stable"), np.argsort(cu[:, 77], kind="stable"))


def test_score_degenerate_inputs():
    wl = _wl_with_q(np.zeros((1, 2, 128), np.float32), Hkv=1)
    st = _store_from(np.full((5, 128), 7), 1.0, [0, 5])
    scores, ex = O.score(wl, st)
    assert not scores.any() and ex[0] == 0           # zero query: all weights zero
    q = np.ones((1, 2, 128), np.float32)
    scores, _ = O.score(_wl_with_q(q, 1), st)
    assert len(set(scores.tolist())) == 1            # equal codes => equal scores
    st0 = _store_from(np.full((5, 128), 7), 0.0, [0, 5])
    scores, ex = O.score(_wl_with_q(q, 1), st0)
    assert not scores.any() and ex[0] == 0           # zero scale (constant channels)


# ------------------------------------------------------------------ O5 Top-K
def _topk(scores, B, T, N=None, stride=None):
    scores = np.asarray(scores, np.int32)
    N = len(scores) if N is None else N
    off = np.array([0, N], np.int64)
    stride = max(N, 1) if stride is None else stride
    idx, cnt = O.topk_raw(1, 1, off, [B], [T], scores, stride)
    return idx[0], int(cnt[0])


def test_topk_matches_lexsort():
    rng = np.random.default_rng(4)
    for N, B, T in [(1, 8, 8), (7, 8, 16), (100, 16, 200), (513, 8, 512), (2048, 32, 4096), (300, 64, 1)]:
        scores = rng.integers(-50, 50, size=N).astype(np.int32)       # many ties
        idx, cnt = _topk(scores, B, T)
        K = min(N, -(-T // B))
        assert cnt == K
        want = np.sort(np.lexsort((np.arange(N), -scores.astype(np.int64)))[:K])
        assert np.array_equal(idx[:K], want)
        assert np.all(idx[K:] == -1)


def test_topk_budget_rule():
    # K = ceil(T/B): K*B >= T > (K-1)*B, clamped to the number of blocks (Sec. 3.4, kernel 2)
    for B in (8, 16, 32, 64, 128):
        for T in (1, 7, 8, 9, 100, 512, 4096, 5000):
            _, cnt = _topk(np.zeros(4096, np.int32), B, T)
            K = cnt
            if K < 4096:
                assert K * B >= T and (K - 1) * B < T
    _, cnt = _topk(np.zeros(10, np.int32), 8, 10 ** 6)
    assert cnt == 10


def test_topk_special_cases():
    s = np.array([5, 9, 9, 1, 9, 0], np.int32)
    idx, cnt = _topk(s, 8, 8)                        # K = 1: first arg-max
    assert cnt == 1 and idx[0] == 1
    idx, cnt = _topk(np.full(12, 3, np.int32), 8, 40)
    assert cnt == 5 and list(idx[:5]) == [0, 1, 2, 3, 4]        # all equal: lowest indices
    idx, cnt = _topk(s, 8, 1000)
    assert cnt == 6 and list(idx[:6]) == [0, 1, 2, 3, 4, 5]     # K >= N: everything
    idx, cnt = _topk(np.array([-2 ** 31, 2 ** 31 - 1, 0, -1], np.int64).astype(np.int32), 8, 16)
    assert list(idx[:2]) == [1, 2]                   # full int32 range, no overflow in the compare


def test_topk_exhaustive_tiny():
    # every score vector over {0,1,2} of length <= 6, every K: the chosen set must dominate the
    # rest under (score desc, index asc) and be listed in ascending index order
    for n in range(1, 7):
        for vec in itertools.product((0, 1, 2), repeat=n):
            for K in range(1, n + 1):
                idx, cnt = _topk(np.array(vec, np.int32), 1, K)
                assert cnt == K
                chosen = list(idx[:K])
                assert chosen == sorted(set(chosen)) and all(0 <= j < n for j in chosen)
                rest = [j for j in range(n) if j not in chosen]
                for i in chosen:
                    for j in rest:
                        assert (vec[i], -i) > (vec[j], -j)


# ------------------------------------------------------------------ O6 attention
def _numpy_attention(wl, tokens_of):
    """Eq. (1) in fp64 with numpy, over tokens_of(b, h) (an index array) for every query head."""
    sm = 1.0 / np.sqrt(wl.head_dim)
    q = synth.bits_to_f32(wl.q, wl.dtype).astype(np.float64)
    out = np.zeros((wl.batch, wl.num_q_heads, wl.head_dim))
    lse = np.zeros((wl.batch, wl.num_q_heads))
    G = wl.group
    for b in range(wl.batch):
        for h in range(wl.num_kv_heads):
            tok = tokens_of(b, h)
            K = wl.key_rows(b, h).astype(np.float64)[tok]
            V = wl.value_rows(b, h).astype(np.float64)[tok]
            for g in range(G):
                z = (K @ q[b, h * G + g]) * sm
                m = z.max()
                e = np.exp(z - m)
                out[b, h * G + g] = (e / e.sum()) @ V
                lse[b, h * G + g] = m + np.log(e.sum())
    return out, lse


@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
def test_full_budget_reproduces_dense_softmax_attention(dtype):
    wl = synth.tiny_workload(seed=11, dtype=dtype, Bt=2, Hq=8, Hkv=2, P=16, seq_lens=(75, 128),
                             block_size=(8, 32), budget=(10 ** 6, 10 ** 6))
    st = O.build_centroids(wl)
    r = O.decode_step(wl, st)
    want, want_lse = _numpy_attention(wl, lambda b, h: np.arange(int(wl.seq_lens[b])))
    assert np.abs(r["out"] - want).max() < 1e-12
    assert np.abs(r["lse"] - want_lse).max() < 1e-12
    dense, dense_lse = O.dense_attention(wl)
    assert np.abs(dense - want).max() < 1e-12 and np.abs(dense_lse - want_lse).max() < 1e-12


def test_sparse_attention_equals_numpy_over_selected_tokens_incl_partial_block():
    wl = synth.tiny_workload(seed=12, Bt=2, Hq=6, Hkv=2, P=16, seq_lens=(75, 41), block_size=(8, 16),
                             budget=(24, 24))
    st = O.build_centroids(wl)
    r = O.decode_step(wl, st)
    # force the trailing partial block into every selection
    sel, cnt = r["sel_idx"].copy(), r["sel_cnt"].copy()
    for s in range(len(cnt)):
        b, h = divmod(s, 2)
        last = -(-int(wl.seq_lens[b]) // int(wl.block_size[h])) - 1
        if last not in sel[s, :cnt[s]]:
            sel[s, cnt[s] - 1] = last
    out, lse = O.sparse_attention(wl, sel, cnt)

    def toks(b, h):
        s = b * 2 + h
        B, L = int(wl.block_size[h]), int(wl.seq_lens[b])
        return np.concatenate([np.arange(j * B, min((j + 1) * B, L)) for j in sel[s, :cnt[s]]])

    want, want_lse = _numpy_attention(wl, toks)
    assert np.abs(out - want).max() < 1e-12 and np.abs(lse - want_lse).max() < 1e-12


def test_attention_closed_forms():
    wl = synth.tiny_workload(seed=13, Bt=1, Hq=4, Hkv=2, P=16, seq_lens=(64,), block_size=(8, 8), budget=(8,))
    # (i) a single selected token (1-token trailing block): out = that value, lse = its logit
    wl1 = synth.tiny_workload(seed=13, Bt=1, Hq=4, Hkv=2, P=16, seq_lens=(65,), block_size=(8, 8), budget=(8,))
    sel = np.full((2, 4), -1, np.int32); sel[:, 0] = 8
    out, lse = O.sparse_attention(wl1, sel, np.array([1, 1], np.int32))
    for h in range(2):
        v = wl1.value_rows(0, h)[64].astype(np.float64)
        k = wl1.key_rows(0, h)[64].astype(np.float64)
        for g in range(2):
            assert np.array_equal(out[0, h * 2 + g], v)
            qv = synth.bits_to_f32(wl1.q, wl1.dtype)[0, h * 2 + g].astype(np.float64)
            assert abs(lse[0, h * 2 + g] - (qv @ k) / np.sqrt(128)) < 1e-12
    # (ii) identical keys: uniform weights, out = mean of the selected values
    wl.k_cache[:] = wl.k_cache[0, 0, 0]
    sel = np.array([[1, 5, -1, -1], [0, 7, -1, -1]], np.int32)
    out, _ = O.sparse_attention(wl, sel, np.array([2, 2], np.int32))
    for h in range(2):
        V = wl.value_rows(0, h).astype(np.float64)
        tok = np.concatenate([np.arange(j * 8, j * 8 + 8) for j in sel[h, :2]])
        for g in range(2):
            assert np.abs(out[0, h * 2 + g] - V[tok].mean(axis=0)).max() < 1e-13
    # (iii) empty selection
    out, lse = O.sparse_attention(wl, sel, np.array([0, 2], np.int32))
    assert not out[0, :2].any() and np.all(np.isneginf(lse[0, :2]))


def test_attention_invariances_and_lse_merge():
    a = synth.tiny_workload(seed=14, shuffle_pages=False, Bt=2, Hq=8, Hkv=2, P=16, seq_lens=(96, 70),
                            block_size=(8, 32), budget=(40, 40))
    st = O.build_centroids(a)
    r = O.decode_step(a, st)
    # physical page permutation changes nothing (block -> page mapping moves no data, Sec. 3.4 kernel 3)
    b = synth.tiny_workload(seed=14, shuffle_pages=False, Bt=2, Hq=8, Hkv=2, P=16, seq_lens=(96, 70),
                            block_size=(8, 32), budget=(40, 40))
    perm = np.random.default_rng(2).permutation(a.num_pages)
    b.k_cache, b.v_cache = a.k_cache[perm], a.v_cache[perm]
    b.page_table = np.argsort(perm)[a.page_table].astype(np.int32)
    rb = O.decode_step(b, O.build_centroids(b))
    assert np.array_equal(r["sel_idx"], rb["sel_idx"]) and np.array_equal(r["out"], rb["out"])
    # order of the index list does not matter (up to fp64 summation order)
    sel, cnt = r["sel_idx"].copy(), r["sel_cnt"]
    for s in range(len(cnt)):
        sel[s, :cnt[s]] = sel[s, :cnt[s]][::-1]
    out_rev, lse_rev = O.sparse_attention(a, sel, cnt)
    assert np.abs(out_rev - r["out"]).max() < 1e-13 and np.abs(lse_rev - r["lse"]).max() < 1e-13
    # split-K: any partition of the selection, merged by the log-sum-exp rule, equals the unsplit result
    half = np.maximum(cnt // 2, 1)
    s1, c1 = r["sel_idx"].copy(), half.astype(np.int32)
    s2 = np.full_like(s1, -1); c2 = (cnt - half).astype(np.int32)
    for s in range(len(cnt)):
        s2[s, :c2[s]] = r["sel_idx"][s, half[s]:cnt[s]]
    o1, l1 = O.sparse_attention(a, s1, c1)
    o2, l2 = O.sparse_attention(a, s2, c2)
    m = np.maximum(l1, l2)
    w1, w2 = np.exp(l1 - m), np.exp(l2 - m)
    merged = (o1 * w1[..., None] + o2 * w2[..., None]) / (w1 + w2)[..., None]
    assert np.abs(merged - r["out"]).max() < 1e-12
    assert np.abs(m + np.log(w1 + w2) - r["lse"]).max() < 1e-12


def test_attention_recall_matches_numpy_definition():
    wl = synth.make_workload(1, context=1024, budget=128)
    st = O.build_centroids(wl)
    r = O.decode_step(wl, st)
    rec = O.attention_recall(wl, r["sel_idx"], r["sel_cnt"])
    q = synth.bits_to_f32(wl.q, wl.dtype).astype(np.float64)
    for h in (0, 3, 7):
        K = wl.key_rows(0, h).astype(np.float64)
        B = int(wl.block_size[h])
        chosen = np.zeros(len(K), bool)
        for j in r["sel_idx"][h, :r["sel_cnt"][h]]:
            chosen[j * B:(j + 1) * B] = True
        for g in range(wl.group):
            z = K @ q[0, h * wl.group + g] / np.sqrt(128)
            a = np.exp(z - z.max()); a /= a.sum()
            assert abs(rec[0, h * wl.group + g] - a[chosen].sum()) < 1e-12
    assert 0.0 <= O.planted_recall(wl, r["sel_idx"], r["sel_cnt"]) <= 1.0


def test_selected_token_count_equals_budget():
    # footnote of Sec. 2.3: the selected blocks hold the budgeted number of tokens
    wl = synth.make_workload(3, context=16384, budget=4096)
    st = O.build_centroids(wl)
    r = O.decode_step(wl, st)
    for h in range(8):
        assert r["sel_cnt"][h] * int(wl.block_size[h]) == 4096


def test_planted_heavy_tokens_are_found():
    # sanity of the workload recipes, not of the oracle: the planted keys dominate attention and
    # fine-grained heads recover them
    wl = synth.make_workload(1)
    r = O.decode_step(wl, O.build_centroids(wl))
    assert O.planted_recall(wl, r["sel_idx"], r["sel_cnt"]) > 0.6
    dense, _ = O.dense_attention(wl)
    assert np.isfinite(dense).all()
