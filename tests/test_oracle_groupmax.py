"""Pins for the group-maximum score (one selection per KV head, ranked by max_g q_g . c^_j): the
oracle function against things it does not compute itself."""
import copy

import numpy as np

from oracle import oracle as O
from paper_2605_12110_amd import synth


def _wl(seed=3, **kw):
    return synth.tiny_workload(seed=seed, Bt=2, Hq=8, Hkv=2, P=16, seq_lens=(301, 512), block_size=(8, 32),
                               budget=(64, 96), **kw)


def _codes(st):
    c = st.codes
    out = np.empty((c.shape[0], c.shape[1] * 2), np.int64)
    out[:, 0::2] = c & 15
    out[:, 1::2] = c >> 4
    return out


def test_scores_are_the_integer_maximum_of_the_reported_heads():
    wl = _wl()
    st = O.build_centroids(wl)
    s, ex, wq, zq = O.score_groupmax(wl, st, want_weights=True)
    codes = _codes(st)
    for seg in range(wl.batch * wl.num_kv_heads):
        blk = codes[st.off[seg]:st.off[seg + 1]]                           # [N, d]
        per_head = blk @ wq[seg].astype(np.int64).T + zq[seg].astype(np.int64)[None, :]
        assert np.array_equal(per_head.max(axis=1), s[st.off[seg]:st.off[seg + 1]].astype(np.int64))
        assert np.abs(wq[seg]).max() <= 32768 and np.abs(wq[seg]).max() >= 16384


def test_offsets_are_the_pairwise_binary32_sums_on_the_groups_scale():
    """zq recomputed with numpy binary32 in the stated order: pairwise inside runs of 16 channels,
    runs added in order; then scaled by the group's exponent and rounded."""
    wl = _wl(seed=9, dtype=synth.BF16)
    st = O.build_centroids(wl)
    _, ex, _, zq = O.score_groupmax(wl, st, want_weights=True)
    G, d = wl.group, wl.head_dim
    q32 = synth.bits_to_f32(wl.q, wl.dtype)
    for seg in range(wl.batch * wl.num_kv_heads):
        b, h = divmod(seg, wl.num_kv_heads)
        for g in range(G):
            prod = (q32[b, h * G + g].astype(np.float32) * st.qmin[seg].astype(np.float32)).astype(np.float32)
            runs = prod.reshape(d // 16, 16)
            while runs.shape[1] > 1:
                runs = (runs[:, 0::2] + runs[:, 1::2]).astype(np.float32)
            z = np.float32(runs[0, 0])
            for k in range(1, d // 16):
                z = np.float32(z + runs[k, 0])
            want = int(np.clip(np.rint(np.float32(np.ldexp(z, -int(ex[seg])))), -2.0 ** 30, 2.0 ** 30))
            assert int(zq[seg, g]) == want


def test_offsets_equal_exact_rational_arithmetic_where_no_summation_order_can_matter():
    """The binary32 sum of the zero-point products has a stated order (a reading, for reproducibility),
    which the test above restates.  This one does not: queries and zero points are small dyadic
    numbers, so every product and every partial sum in ANY order is exact in binary32, and z_g must
    equal the sum in exact rational arithmetic; scaled by the group's exponent and rounded half to even
    it must give the reported offsets.  A dropped channel, a wrong sign or head, or the scale of another
    head fails here whatever the order."""
    from fractions import Fraction
    wl = _wl(seed=21)
    rng = np.random.default_rng(22)
    q = rng.integers(-8, 9, size=wl.q.shape).astype(np.float32) / 4.0            # multiples of 1/4 in [-2, 2]
    wl.q = synth.f32_to_bits(q, wl.dtype)
    st = O.build_centroids(wl)
    st.qmin[:] = (rng.integers(-64, 65, size=st.qmin.shape) / 8.0).astype(np.float32)   # multiples of 1/8 in [-8, 8]
    st.qscale[:] = (2.0 ** rng.integers(-6, -2, size=st.qscale.shape)).astype(np.float32)
    s, ex, wq, zq = O.score_groupmax(wl, st, want_weights=True)
    G, d = wl.group, wl.head_dim
    for seg in range(wl.batch * wl.num_kv_heads):
        b, h = divmod(seg, wl.num_kv_heads)
        for g in range(G):
            z = sum(Fraction(float(q[b, h * G + g, c])) * Fraction(float(st.qmin[seg, c])) for c in range(d))
            scaled = z / Fraction(2) ** int(ex[seg])
            lo = scaled.numerator // scaled.denominator                          # floor
            frac = scaled - lo
            want = lo + (1 if frac > Fraction(1, 2) or (frac == Fraction(1, 2) and lo % 2 == 1) else 0)
            want = max(-2 ** 30, min(2 ** 30, want))
            assert int(zq[seg, g]) == want, (seg, g)
            # and the weights on the same scale, exactly
            for c in range(0, d, 17):
                w = Fraction(float(q[b, h * G + g, c])) * Fraction(float(st.qscale[seg, c])) / Fraction(2) ** int(ex[seg])
                assert w.denominator == 1 and int(wq[seg, g, c]) == w.numerator


def test_score_is_within_the_rounding_bound_of_the_fp64_maximum_over_dequantized_centroids():
    wl = _wl(seed=21)
    st = O.build_centroids(wl)
    s, ex = O.score_groupmax(wl, st)
    deq = O.dequantize(st.off, st.codes, st.qscale, st.qmin).astype(np.float64)
    G, d = wl.group, wl.head_dim
    q64 = synth.bits_to_f32(wl.q, wl.dtype).astype(np.float64)
    for seg in range(wl.batch * wl.num_kv_heads):
        b, h = divmod(seg, wl.num_kv_heads)
        qs = q64[b, h * G:(h + 1) * G]                                          # [G, d]
        exact = (deq[st.off[seg]:st.off[seg + 1]] @ qs.T).max(axis=1)
        got = np.ldexp(s[st.off[seg]:st.off[seg + 1]].astype(np.float64), int(ex[seg]))
        ulp = 2.0 ** int(ex[seg])
        slack = 1e-5 * (np.abs(qs) @ (np.abs(st.qmin[seg]) + 15 * np.abs(st.qscale[seg])).astype(np.float64)).max()
        assert np.abs(got - exact).max() <= (d * 7.5 + 0.5) * ulp + slack


def test_a_single_head_group_ranks_like_the_default_score():
    wl = synth.tiny_workload(seed=4, Bt=2, Hq=2, Hkv=2, P=16, seq_lens=(400, 90), block_size=(8, 16), budget=(64, 32))
    st = O.build_centroids(wl)
    s_max, ex_max, _, zq = O.score_groupmax(wl, st, want_weights=True)
    s_sum, ex_sum = O.score(wl, st)
    assert np.array_equal(ex_max, ex_sum)
    for seg in range(wl.batch * wl.num_kv_heads):
        diff = s_max[st.off[seg]:st.off[seg + 1]].astype(np.int64) - s_sum[st.off[seg]:st.off[seg + 1]]
        assert np.all(diff == int(zq[seg, 0]))


def test_equal_heads_give_the_single_heads_score_plus_its_offset():
    wl = _wl(seed=5)
    G = wl.group
    wl.q = np.repeat(wl.q[:, ::G], G, axis=1)
    st = O.build_centroids(wl)
    s_max, ex_max, _, zq = O.score_groupmax(wl, st, want_weights=True)
    one = copy.copy(wl)
    one.num_q_heads = wl.num_kv_heads
    one.q = np.ascontiguousarray(wl.q[:, ::G])
    s_one, ex_one = O.score(one, st)
    assert np.array_equal(ex_max, ex_one)
    for seg in range(wl.batch * wl.num_kv_heads):
        assert np.all(zq[seg] == zq[seg, 0])
        assert np.array_equal(s_max[st.off[seg]:st.off[seg + 1]].astype(np.int64),
                              s_one[st.off[seg]:st.off[seg + 1]].astype(np.int64) + int(zq[seg, 0]))


def test_opposite_one_hot_heads_rank_blocks_by_the_magnitude_of_that_channel():
    """q_0 = +e_c, q_1 = -e_c: the two heads score a block +c^_jc and -c^_jc, the maximum is |c^_jc|.
    The zero-point offset decides that ranking: without it the order would be that of the codes."""
    wl = synth.tiny_workload(seed=6, Bt=1, Hq=2, Hkv=1, P=16, seq_lens=(1024,), block_size=(8,), budget=(64,))
    ch = 17
    q = np.zeros((1, 2, wl.head_dim), np.float32)
    q[0, 0, ch], q[0, 1, ch] = 1.0, -1.0
    wl.q = synth.f32_to_bits(q, wl.dtype)
    st = O.build_centroids(wl)
    s, ex = O.score_groupmax(wl, st)
    deq = O.dequantize(st.off, st.codes, st.qscale, st.qmin).astype(np.float64)[:, ch]
    got = np.ldexp(s.astype(np.float64), int(ex[0]))
    assert np.abs(got - np.abs(deq)).max() <= 8.5 * 2.0 ** int(ex[0]) + 1e-6
    assert deq.min() < 0 < deq.max()                     # the channel changes sign: codes alone would misrank
    order = np.argsort(-s, kind="stable")
    assert np.all(np.diff(np.abs(deq)[order]) <= 17 * 2.0 ** int(ex[0]))


def test_degenerate_queries_score_zero():
    wl = _wl(seed=8)
    wl.q = np.zeros_like(wl.q)
    st = O.build_centroids(wl)
    s, ex = O.score_groupmax(wl, st)
    assert not s.any() and not ex.any()


def test_step_with_the_group_maximum_is_dense_when_the_budget_covers_the_context():
    wl = _wl(seed=10)
    wl.budget = np.array([4096, 4096], np.int32)
    r = O.decode_step(wl, O.build_centroids(wl), group_max=True)
    dense, lse = O.dense_attention(wl)
    assert np.abs(r["out"] - dense).max() < 1e-12 and np.abs(r["lse"] - lse).max() < 1e-12
