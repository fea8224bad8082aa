"""Pins for the oracle's centroid build and INT4 quantization (no GPU).

Each check compares the C oracle with something that is not the oracle: numpy fp64
means, numpy's own fp16 widening, closed forms (constant keys, single-key blocks),
invariants the paper fixes (mean pooling, Sec. 2.2; one scale and zero-point per channel,
16 levels, Sec. 3.3; prefix-sum segment layout, Sec. 3.4 kernel 1) and brute force on
tiny inputs.
"""
import numpy as np
import pytest

from oracle import oracle as O
from paper_2605_12110_amd import synth


def _codes_unpacked(codes):
    lo = codes & 15
    hi = codes >> 4
    return np.stack([lo, hi], axis=-1).reshape(codes.shape[0], -1)


def test_widening_matches_numpy_for_every_f16_pattern():
    # block size 1 => each centroid is exactly one key: exposes the oracle's fp16 widening
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    finite = np.isfinite(bits.view(np.float16))
    bits = bits[finite]
    n = (len(bits) // 128) * 128
    bits = bits[:n]
    wl = synth.tiny_workload(Bt=1, Hq=1, Hkv=1, P=16, seq_lens=(n // 128,), block_size=(1,), budget=(1,),
                             shuffle_pages=False, extra_pages=0)
    rows = bits.reshape(-1, 128)
    pad = wl.k_cache.reshape(-1, 128).shape[0] - rows.shape[0]
    wl.k_cache = np.concatenate([rows, np.zeros((pad, 128), np.uint16)]).reshape(wl.k_cache.shape)
    off = O.offsets(wl)
    cent = O.centroids(wl, off)
    want = rows.view(np.float16).astype(np.float32).view(np.uint32)
    nz = want != 0x80000000          # 0 + (-0) = +0 in the running sum
    assert np.array_equal(cent.view(np.uint32)[nz], want[nz])


def test_widening_bf16_matches_shift():
    rng = np.random.default_rng(5)
    bits = rng.integers(0, 65536, size=(64, 128), dtype=np.uint32).astype(np.uint16)
    f = synth.bits_to_f32(bits, synth.BF16)
    bits = bits[np.isfinite(f).all(axis=1)]
    L = bits.shape[0]
    wl = synth.tiny_workload(dtype=synth.BF16, Bt=1, Hq=1, Hkv=1, P=16, seq_lens=(L,), block_size=(1,),
                             budget=(1,), shuffle_pages=False, extra_pages=0)
    kc = wl.k_cache.reshape(-1, 128)
    kc[:L] = bits
    cent = O.centroids(wl, O.offsets(wl))
    want = (bits.astype(np.uint32) << 16)
    got = cent.view(np.uint32)
    nz = want != 0x80000000          # 0 + (-0) = +0 in the running sum
    assert np.array_equal(got[nz], want[nz])


def test_offsets_are_prefix_sums_of_ceil_L_over_B():
    wl = synth.tiny_workload(Bt=3, Hkv=4, Hq=8, seq_lens=(1, 100, 257), block_size=(8, 16, 32, 128),
                             budget=(8, 8, 8))
    off = O.offsets(wl)
    n = np.diff(off).reshape(3, 4)
    for b, L in enumerate((1, 100, 257)):
        for h, B in enumerate((8, 16, 32, 128)):
            assert n[b, h] == -(-L // B)
    assert off[0] == 0 and off[-1] == n.sum()


def test_paper_size_arithmetic_from_golden():
    # Sec. 1: a single 128K request on Llama-3.1-8B holds 16 GB of KV cache
    vals = {}
    with open(__file__.rsplit("/", 1)[0] + "/golden/paper_sizes.txt") as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split("=")
                vals[k.strip()] = int(v)
    total = (vals["context"] * vals["layers"] * vals["kv_heads"] * vals["head_dim"] * 2 * vals["bytes_per_elem"])
    assert total == vals["kv_cache_gib"] * 2 ** 30
    wl3_bytes_per_layer = total // vals["layers"]
    assert wl3_bytes_per_layer == 512 * 2 ** 20


@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
def test_centroid_is_mean_of_its_keys(dtype):
    wl = synth.tiny_workload(seed=3, dtype=dtype, Bt=2, Hkv=2, Hq=4, P=16, seq_lens=(75, 128),
                             block_size=(8, 32), budget=(8, 8))
    off = O.offsets(wl)
    cent = O.centroids(wl, off)
    for b in range(wl.batch):
        for h in range(wl.num_kv_heads):
            keys = wl.key_rows(b, h).astype(np.float64)
            B = int(wl.block_size[h])
            s = b * wl.num_kv_heads + h
            N = -(-keys.shape[0] // B)
            for j in range(N):
                blk = keys[j * B:(j + 1) * B]
                want = blk.mean(axis=0)
                got = cent[off[s] + j].astype(np.float64)
                n = blk.shape[0]
                tol = (n + 1) * 2.0 ** -24 * np.abs(blk).sum(axis=0).max()
                assert np.abs(got - want).max() <= tol


def test_constant_keys_and_single_key_blocks_are_exact():
    wl = synth.tiny_workload(seed=4, Bt=1, Hkv=2, Hq=2, P=16, seq_lens=(33,), block_size=(8, 16), budget=(8,))
    row = synth.f32_to_bits(np.linspace(-2, 2, 128, dtype=np.float32), wl.dtype)
    wl.k_cache[:, 0] = row                       # head 0: every key identical
    off = O.offsets(wl)
    cent = O.centroids(wl, off)
    want = synth.bits_to_f32(row, wl.dtype)
    for j in range(off[1] - off[0]):             # includes the 1-token trailing block (33 = 4*8+1)
        assert np.array_equal(cent[off[0] + j], want)
    # head 1: trailing block of 33 tokens with B=16 holds exactly token 32
    assert np.array_equal(cent[off[2] - 1], wl.key_rows(0, 1)[32])


def test_build_is_invariant_under_physical_page_permutation():
    a = synth.tiny_workload(seed=7, shuffle_pages=False, seq_lens=(80, 45))
    b = synth.tiny_workload(seed=7, shuffle_pages=False, seq_lens=(80, 45))
    perm = np.random.default_rng(1).permutation(a.num_pages)
    inv = np.argsort(perm)
    b.k_cache = a.k_cache[perm]                  # physical page p of b holds a's page perm[p]
    b.v_cache = a.v_cache[perm]
    b.page_table = inv[a.page_table].astype(np.int32)
    sa, sb = O.build_centroids(a), O.build_centroids(b)
    assert np.array_equal(sa.cent.view(np.uint32), sb.cent.view(np.uint32))
    assert np.array_equal(sa.codes, sb.codes)
    assert np.array_equal(sa.qscale, sb.qscale) and np.array_equal(sa.qmin, sb.qmin)


def test_quantization_closed_forms():
    wl = synth.make_workload(1, context=1024)
    st = O.build_centroids(wl)
    codes = _codes_unpacked(st.codes)
    assert codes.min() >= 0 and codes.max() <= 15
    deq = O.dequantize(st.off, st.codes, st.qscale, st.qmin)
    for s in range(len(st.off) - 1):
        lo, hi = st.off[s], st.off[s + 1]
        c = st.cent[lo:hi]
        # one (scale, min) per channel shared by all blocks; range = exact min/max; 16 levels
        assert np.array_equal(st.qmin[s], c.min(axis=0))
        rng = (c.max(axis=0) - c.min(axis=0)).astype(np.float32)
        assert np.array_equal(st.qscale[s], (rng / np.float32(15.0)).astype(np.float32))
        # the channel minimum gets code 0, the maximum code 15
        assert np.all(codes[lo:hi][c.argmin(axis=0), np.arange(128)] == 0)
        assert np.all(codes[lo:hi][c.argmax(axis=0), np.arange(128)] == 15)
        # |dequant - centroid| <= scale/2 (plus a hair for the binary32 roundings)
        err = np.abs(deq[lo:hi].astype(np.float64) - c.astype(np.float64))
        assert np.all(err <= st.qscale[s].astype(np.float64) * 0.5 * (1 + 2.0 ** -18) + 1e-12)
        # and the code is the nearest level: independent fp64 rounding agrees except at exact ties
        y = (c.astype(np.float64) - st.qmin[s].astype(np.float64)) / np.maximum(rng.astype(np.float64), 1e-300) * 15.0
        near = np.abs(codes[lo:hi] - y) <= 0.5 + 1e-5
        assert near.all()


def test_quantization_round_trip_is_idempotent():
    wl = synth.make_workload(1, context=2048)
    st = O.build_centroids(wl)
    deq = O.dequantize(st.off, st.codes, st.qscale, st.qmin)
    again = O.quantize(st.off, deq, st.qmin, st.qinv)
    assert np.array_equal(again, st.codes)


def test_constant_channel_is_exact_with_zero_scale():
    wl = synth.tiny_workload(seed=2, Bt=1, Hkv=1, Hq=1, P=16, seq_lens=(64,), block_size=(8,), budget=(8,))
    kc = wl.k_cache
    kc[..., 5] = synth.f32_to_bits(np.float32(0.75), wl.dtype)      # channel 5 constant everywhere
    st = O.build_centroids(wl)
    assert np.all(st.qscale[:, 5] == 0) and np.all(st.qinv[:, 5] == 0) and np.all(st.qmin[:, 5] == 0.75)
    assert np.all(_codes_unpacked(st.codes)[:, 5] == 0)
    assert np.all(O.dequantize(st.off, st.codes, st.qscale, st.qmin)[:, 5] == 0.75)


def test_code_packing_low_nibble_is_even_channel_hand_case():
    # 16 centroids whose channel c takes the values j*(c+1), j = 0..15: code of block j is j in
    # every channel, so byte i of block j must be (j<<4)|j; then break symmetry on channel 3.
    off = np.array([0, 16], dtype=np.int64)
    cent = (np.arange(16, dtype=np.float32)[:, None] * (np.arange(128, dtype=np.float32)[None, :] + 1)).copy()
    qscale, qmin, qinv = O.quant_params(off, cent)
    codes = O.quantize(off, cent, qmin, qinv)
    assert np.array_equal(codes, np.repeat(((np.arange(16) << 4) | np.arange(16)).astype(np.uint8)[:, None], 64, 1))
    assert np.array_equal(qscale[0], (np.arange(128) + 1).astype(np.float32))
    cent[:, 3] = cent[::-1, 3].copy()            # channel 3 (odd => high nibble of byte 1) reversed
    qscale, qmin, qinv = O.quant_params(off, cent)
    codes = O.quantize(off, cent, qmin, qinv)
    j = np.arange(16)
    assert np.array_equal(codes[:, 1], (((15 - j) << 4) | j).astype(np.uint8))
    assert np.array_equal(codes[:, 0], ((j << 4) | j).astype(np.uint8))


def test_rounding_is_half_to_even_hand_case():
    # two-level channel: values 0 and 15 fix scale 1; then 0.5 -> 0, 1.5 -> 2, 2.5 -> 2, 3.5 -> 4
    vals = np.array([0, 15, 0.5, 1.5, 2.5, 3.5, 14.5, 7.49, 7.51], dtype=np.float32)
    off = np.array([0, len(vals)], dtype=np.int64)
    cent = np.zeros((len(vals), 128), np.float32)
    cent[:, 0] = vals
    cent[:, 1] = -vals                          # min = -15: (-v + 15) has the mirrored ties
    qscale, qmin, qinv = O.quant_params(off, cent)
    codes = _codes_unpacked(O.quantize(off, cent, qmin, qinv))
    assert list(codes[:, 0]) == [0, 15, 0, 2, 2, 4, 14, 7, 8]
    assert list(codes[:, 1]) == [15, 0, 14, 14, 12, 12, 0, 8, 7]


def test_int4_ranking_recall_against_unquantized_centroids():
    # Sec. 3.3: INT4 asymmetric per-channel keeps Top-K recall above 0.9
    for cfg, ctx in ((1, 4096), (2, 8192), (3, 16384)):
        wl = synth.make_workload(cfg, context=ctx, batch=1)
        st = O.build_centroids(wl)
        scores, _ = O.score(wl, st)
        sel, cnt = O.topk(wl, st.off, scores)
        G = wl.group
        q = synth.bits_to_f32(wl.q, wl.dtype).astype(np.float64)
        hit = tot = 0
        for s in range(len(st.off) - 1):
            b, h = divmod(s, wl.num_kv_heads)
            u = q[b, h * G:(h + 1) * G].sum(axis=0)
            exact = st.cent[st.off[s]:st.off[s + 1]].astype(np.float64) @ u
            k = int(cnt[s])
            ref = set(np.argsort(-exact, kind="stable")[:k].tolist())
            hit += len(ref & set(sel[s, :k].tolist()))
            tot += k
        assert hit / tot >= 0.9, (cfg, hit / tot)
