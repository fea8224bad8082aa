"""Pins for the oracle's quantization variants (Sec. 3.3 design space; no GPU): the 4-bit asymmetric
variant must be the store's own quantizer bit for bit, every variant must meet its half-step error
bound and reach its extreme codes, symmetric stores are zero-centred, and the score on a variant
must be the integer dot with the signed codes."""
import numpy as np
import pytest

from oracle import oracle as O
from paper_2605_12110_amd import synth


def _unpack(codes):
    return np.stack([codes & 15, codes >> 4], axis=-1).reshape(codes.shape[0], -1)


def test_four_bit_asymmetric_variant_is_the_stores_quantizer():
    wl = synth.make_workload(1, context=2048)
    st = O.build_centroids(wl)
    qscale, qmin, codes, zero = O.quantize_variant(st.off, st.cent, 4, False)
    assert zero == 0 and np.array_equal(qscale, st.qscale) and np.array_equal(qmin, st.qmin)
    assert np.array_equal(codes, _unpack(st.codes))
    s1, e1 = O.score(wl, st)
    s2, e2 = O.score_variant(wl, st.off, codes, qscale, zero)
    assert np.array_equal(s1, s2) and np.array_equal(e1, e2)


@pytest.mark.parametrize("bits", [2, 4, 8])
@pytest.mark.parametrize("symmetric", [False, True])
def test_every_variant_meets_its_half_step_bound_and_reaches_its_extremes(bits, symmetric):
    wl = synth.make_workload(2, context=1024, batch=1)
    st = O.build_centroids(wl)
    qscale, qmin, codes, zero = O.quantize_variant(st.off, st.cent, bits, symmetric)
    top = (1 << (bits - 1)) - 1 if symmetric else (1 << bits) - 1
    for s in range(len(st.off) - 1):
        x = st.cent[st.off[s]:st.off[s + 1]].astype(np.float64)
        c = codes[st.off[s]:st.off[s + 1]].astype(np.float64) - zero
        sc, mn = qscale[s].astype(np.float64), qmin[s].astype(np.float64)
        assert np.all(np.abs(c * sc + mn - x) <= sc / 2 * (1 + 1e-5) + 1e-12)
        if symmetric:
            assert not qmin[s].any() and np.all(np.abs(c) <= top)
            assert np.allclose(sc * top, np.abs(x).max(axis=0), rtol=1e-6)
            assert np.all(np.abs(c).max(axis=0) == top)                # the largest magnitude sits on the last level
        else:
            assert np.all(c.min(axis=0) == 0) and np.all(c.max(axis=0) == top)


def test_score_on_a_symmetric_store_is_the_integer_dot_with_signed_codes():
    q = np.zeros((1, 1, 128), np.float32)
    q[0, 0, :2] = [1.0, -0.5]
    wl = synth.tiny_workload(Bt=1, Hq=1, Hkv=1, P=16, seq_lens=(64,), block_size=(8,), budget=(8,))
    wl.q = synth.f32_to_bits(q, wl.dtype)
    rng = np.random.default_rng(0)
    codes = rng.integers(0, 15, size=(8, 128)).astype(np.uint8)          # stored codes 0..14, zero at 7
    qs = np.ones((1, 128), np.float32)
    off = np.array([0, 8], np.int64)
    scores, ex = O.score_variant(wl, off, codes, qs, 7)
    assert ex[0] == -14
    want = [16384 * (int(c[0]) - 7) - 8192 * (int(c[1]) - 7) for c in codes]
    assert list(scores) == want


def test_ranking_recall_orders_the_variants_as_the_paper_reports():
    """Top-K recall against the unquantized centroids (Sec. 3.3): 2 bits lose the ranking, 8 bits keep
    it, 4-bit asymmetric stays above 0.9 and is not worse than 4-bit symmetric."""
    wl = synth.make_workload(3, context=16384, budget=1024)
    st = O.build_centroids(wl)
    u = synth.bits_to_f32(wl.q, wl.dtype).astype(np.float64).reshape(wl.num_kv_heads, wl.group, 128).sum(axis=1)
    exact = np.concatenate([st.cent[st.off[s]:st.off[s + 1]].astype(np.float64) @ u[s] for s in range(8)])
    key = np.round(exact * 2 ** 20).astype(np.int64).clip(-2 ** 31 + 1, 2 ** 31 - 1).astype(np.int32)
    ref_idx, ref_cnt = O.topk(wl, st.off, key)
    rec = {}
    for bits in (2, 4, 8):
        for sym in (False, True):
            qs, qm, codes, zero = O.quantize_variant(st.off, st.cent, bits, sym)
            sc, _ = O.score_variant(wl, st.off, codes, qs, zero)
            idx, cnt = O.topk(wl, st.off, sc)
            hits = sum(len(set(idx[s, :cnt[s]]) & set(ref_idx[s, :ref_cnt[s]])) for s in range(8))
            rec[(bits, sym)] = hits / ref_cnt.sum()
    assert rec[(4, False)] >= 0.9 and rec[(8, False)] >= 0.98 and rec[(8, True)] >= 0.98
    assert rec[(2, False)] < rec[(4, False)] and rec[(2, True)] < rec[(4, True)]
    assert rec[(4, False)] >= rec[(4, True)] - 0.02
