"""Pins for the oracle's decode-time store maintenance (no GPU): a new token is folded into the
pooled state of its segment's last block and that block's 4-bit row is re-emitted under the
store's frozen ranges.  Pinned to the already pinned rebuild functions (the block value must be
bit-identical to a rebuild's; the row must be what the quantizer gives for that value under the
frozen parameters), to closed forms (clamping, constant keys) and to structural facts (closed rows
never change, a row appears exactly when a block opens)."""
import copy

import numpy as np
import pytest

from oracle import oracle as O
from paper_2605_12110_amd import synth


def _at(wl, lens):
    """The same caches seen at shorter context lengths (the tokens beyond are already in the pages)."""
    v = copy.copy(wl)
    v.seq_lens = np.asarray(lens, np.int32)
    return v


def _unpack(codes):
    return np.stack([codes & 15, codes >> 4], axis=-1).reshape(codes.shape[0], -1).astype(np.int64)


@pytest.mark.parametrize("repr_", [O.MEAN, O.MINMAX])
def test_tail_state_is_the_last_blocks_pooled_value(repr_):
    wl = synth.tiny_workload(seed=61, Bt=3, Hq=4, Hkv=2, P=16, seq_lens=(37, 64, 130), block_size=(8, 32),
                             budget=(8, 8, 8))
    tail = O.tail_state(wl, repr_)
    st = O.build_centroids(wl, repr_)
    for s in range(6):
        b, h = divmod(s, 2)
        L, B = int(wl.seq_lens[b]), int(wl.block_size[h])
        n = L - (L - 1) // B * B
        last = st.cent[st.off[s + 1] - 1]
        if repr_ == O.MEAN:
            assert np.array_equal(tail[s] / np.float32(n), last)      # same single division as the rebuild
        else:
            assert np.array_equal(tail[s], last)


@pytest.mark.parametrize("repr_,dtype", [(O.MEAN, synth.F16), (O.MEAN, synth.BF16), (O.MINMAX, synth.F16)])
def test_appending_token_by_token_tracks_a_rebuild_bit_for_bit_in_value_and_keeps_closed_rows(repr_, dtype):
    full = synth.tiny_workload(seed=62, dtype=dtype, Bt=2, Hq=4, Hkv=2, P=16, seq_lens=(150, 97), block_size=(8, 32),
                               budget=(8, 8))
    start = np.array([150 - 40, 97 - 40], np.int32)
    wl = _at(full, start)
    store = O.build_centroids(wl, repr_)
    frozen_scale, frozen_min = store.qscale.copy(), store.qmin.copy()
    tail = O.tail_state(wl, repr_)
    for step in range(1, 41):
        wl = _at(full, start + step)
        prev = store
        store, values = O.append_token(wl, prev, tail)
        rebuilt = O.build_centroids(wl, repr_)
        assert np.array_equal(store.off, rebuilt.off)                 # tight layout of the new lengths
        assert np.array_equal(tail, O.tail_state(wl, repr_))
        inv = (np.float32(1.0) / np.where(frozen_scale > 0, frozen_scale, np.float32(1))).astype(np.float32)
        inv = np.where(frozen_scale > 0, inv, np.float32(0)).astype(np.float32)
        for s in range(4):
            last = int(store.off[s + 1]) - 1
            # the open block's value is the rebuild's, bit for bit
            assert np.array_equal(values[s], rebuilt.cent[last])
            # closed rows are carried over untouched
            n_closed = last - int(store.off[s])
            assert np.array_equal(store.codes[store.off[s]:last], prev.codes[prev.off[s]:prev.off[s] + n_closed])
            # the re-emitted row = the (pinned) quantizer on that value under the frozen parameters
            one_off = np.array([0, 1], np.int64)
            want = O.quantize(one_off, values[s:s + 1], frozen_min[s:s + 1], inv[s:s + 1])
            assert np.array_equal(store.codes[last:last + 1], want)
        assert np.array_equal(store.qscale, frozen_scale) and np.array_equal(store.qmin, frozen_min)


def test_a_row_appears_exactly_when_a_block_opens_and_holds_the_new_key_alone():
    full = synth.tiny_workload(seed=63, Bt=1, Hq=2, Hkv=1, P=16, seq_lens=(64,), block_size=(8,), budget=(8,))
    wl = _at(full, [40])                                              # 5 complete blocks
    store = O.build_centroids(wl)
    tail = O.tail_state(wl)
    wl = _at(full, [41])
    grown, values = O.append_token(wl, store, tail)
    assert int(grown.off[-1]) == 6 and np.array_equal(grown.codes[:5], store.codes)
    key = full.key_rows(0, 0)[40]
    assert np.array_equal(values[0], key) and np.array_equal(tail[0], key)
    for _ in range(7):                                                # fill the block: no new row
        wl = _at(full, [int(wl.seq_lens[0]) + 1])
        grown, _ = O.append_token(wl, grown, tail)
        assert int(grown.off[-1]) == 6


def test_values_outside_the_frozen_range_clamp_and_inside_it_stay_within_half_a_step():
    full = synth.tiny_workload(seed=64, Bt=1, Hq=2, Hkv=1, P=16, seq_lens=(72,), block_size=(8,), budget=(8,))
    wl = _at(full, [64])
    store = O.build_centroids(wl)
    tail = O.tail_state(wl)
    # token 64 opens block 8: make its key huge on even channels, hugely negative on odd ones
    pg = full.page_table[0, 4]
    big = np.where(np.arange(128) % 2 == 0, 1000.0, -1000.0).astype(np.float32)
    full.k_cache[pg, 0, 0] = synth.f32_to_bits(big, full.dtype)
    wl = _at(full, [65])
    grown, values = O.append_token(wl, store, tail)
    cu = _unpack(grown.codes[8:9])[0]
    assert np.all(cu[0::2] == 15) and np.all(cu[1::2] == 0)
    # an ordinary key inside the range: dequantized value within half a step
    full2 = synth.tiny_workload(seed=64, Bt=1, Hq=2, Hkv=1, P=16, seq_lens=(72,), block_size=(8,), budget=(8,))
    tail = O.tail_state(_at(full2, [64]))
    grown, values = O.append_token(_at(full2, [65]), store, tail)
    cu = _unpack(grown.codes[8:9])[0].astype(np.float64)
    sc, mn = store.qscale[0].astype(np.float64), store.qmin[0].astype(np.float64)
    v = values[0].astype(np.float64)
    inside = (v >= mn) & (v <= mn + 15 * sc)
    assert inside.sum() > 20          # a one-key block often lies outside the range of 8-key means: those clamp
    assert np.all(np.abs(cu * sc + mn - v)[inside] <= sc[inside] / 2 * (1 + 1e-5) + 1e-12)
    assert np.all(cu[v < mn] == 0) and np.all(cu[v > mn + 15 * sc] == 15)


def test_constant_keys_keep_their_code_and_zero_scale_channels_stay_zero():
    full = synth.tiny_workload(seed=65, Bt=1, Hq=2, Hkv=1, P=16, seq_lens=(48,), block_size=(16,), budget=(8,))
    # block 2 (tokens 32..47) holds one key repeated; channel 5 is constant over the whole context
    pg = full.page_table[0, 2]
    full.k_cache[pg, 0, :] = full.k_cache[pg, 0, 0]
    for p in range(3):
        full.k_cache[full.page_table[0, p], 0, :, 5] = full.k_cache[full.page_table[0, 0], 0, 0, 5]
    wl = _at(full, [33])
    store = O.build_centroids(wl)
    assert store.qscale[0, 5] == 0
    tail = O.tail_state(wl)
    row = store.codes[2].copy()
    grown = store
    for L in range(34, 49):
        grown, _ = O.append_token(_at(full, [L]), grown, tail)
        cu_new, cu_old = _unpack(grown.codes[2:3])[0], _unpack(row[None])[0]
        # a mean of equal fp16 keys is the key itself up to the rounding of sum/n: at most one level off
        assert np.all(np.abs(cu_new - cu_old) <= 1) and cu_new[5] == 0


# ------------------------------------------------------------------ the re-ranging signal
def _outside(values, scale, mn):
    """Independent count (numpy, exact rational thresholds in float64): a value is held by a frozen
    range [mn, mn + 15*scale] iff its code rint((v - mn) * (1/scale)) lies in [0, 15]; with the
    binary32 steps of the emitter that is decided here from the binary32 product itself."""
    inv = (np.float32(1.0) / np.where(scale > 0, scale, np.float32(1))).astype(np.float32)
    r = np.rint(((values - mn).astype(np.float32) * inv).astype(np.float32))
    return np.where(scale > 0, (r < 0) | (r > 15), values != mn)


@pytest.mark.parametrize("repr_", [O.MEAN, O.MINMAX])
def test_clamp_counter_counts_completed_blocks_only_and_matches_an_independent_count(repr_):
    full = synth.tiny_workload(seed=66, dtype=synth.BF16, Bt=2, Hq=4, Hkv=2, P=16, seq_lens=(150, 97),
                               block_size=(8, 32), budget=(8, 8))
    # outliers among the tokens to come, so that some completed blocks leave the ranges
    rng = np.random.default_rng(5)
    k32 = synth.bits_to_f32(full.k_cache, full.dtype)
    k32 *= np.where(rng.random(k32.shape) < 0.02, 6.0, 1.0).astype(np.float32)
    full.k_cache[:] = synth.f32_to_bits(k32, full.dtype)
    start = np.array([150 - 70, 97 - 70], np.int32)
    wl = _at(full, start)
    store = O.build_centroids(wl, repr_)
    tail = O.tail_state(wl, repr_)
    clamped = np.zeros(4, np.int32)
    want = np.zeros(4, np.int64)
    for step in range(1, 71):
        wl = _at(full, start + step)
        before = clamped.copy()
        store, values = O.append_token(wl, store, tail, clamped)
        for s in range(4):
            b, h = divmod(s, 2)
            if int(wl.seq_lens[b]) % int(wl.block_size[h]) == 0:          # the token completed its block
                want[s] += int(_outside(values[s], store.qscale[s], store.qmin[s]).sum())
            else:
                assert clamped[s] == before[s]
        assert np.array_equal(clamped, want)
    assert clamped.sum() > 0 and np.all(clamped[[0, 2]] > 0)              # blocks of 8: several completed, some outside


def test_clamp_counter_hand_case_boundaries_and_zero_scale_channels():
    full = synth.tiny_workload(seed=67, Bt=1, Hq=2, Hkv=1, P=8, seq_lens=(24,), block_size=(8,), budget=(8,))
    # blocks 0 and 1 fix the ranges: channel c spans [0, 1.5] (step 0.1), channel 5 is constant 0.25
    k = np.zeros((24, 128), np.float32)
    k[8:16] = 1.5
    k[:16, 5] = 0.25
    # block 2 (one key repeated, so its mean is the key): inside, on both ends, half a step beyond, far out
    last = np.full(128, 0.75, np.float32)
    last[0], last[1] = 0.0, 1.5                       # the ends: codes 0 and 15, held
    last[2] = 1.5390625                               # (v - 0) / 0.1 = 15.39 -> 15, held
    last[3] = 1.5625                                  # 15.625 -> 16: outside
    last[4] = -0.0625                                 # -0.625 -> -1: outside
    last[5] = 0.25                                    # constant channel, same value: held
    last[6] = 100.0                                   # far outside
    k[16:24] = last
    for t in range(24):
        full.k_cache[full.page_table[0, t // 8], 0, t % 8] = synth.f32_to_bits(k[t], full.dtype)
    wl = _at(full, [16])
    store = O.build_centroids(wl)
    assert store.qscale[0, 5] == 0 and store.qmin[0, 5] == np.float32(0.25)
    assert np.all(store.qmin[0, [0, 1, 2, 3, 4, 6]] == 0) and np.allclose(store.qscale[0, :5], 0.1)
    tail = O.tail_state(wl)
    clamped = np.array([7], np.int32)                 # the count is added to what is there
    for L in range(17, 25):
        store, _ = O.append_token(_at(full, [L]), store, tail, clamped)
        assert clamped[0] == (7 if L < 24 else 7 + 3)
    # the same block with the constant channel moved: one more value outside
    k[16:24, 5] = 0.5
    for t in range(16, 24):
        full.k_cache[full.page_table[0, t // 8], 0, t % 8] = synth.f32_to_bits(k[t], full.dtype)
    store = O.build_centroids(wl)
    tail = O.tail_state(wl)
    clamped = np.zeros(1, np.int32)
    for L in range(17, 25):
        store, _ = O.append_token(_at(full, [L]), store, tail, clamped)
    assert clamped[0] == 4
