"""Pins for the oracle's calibration rule (Sec. 3.2, Eq. (2)) and the recall it consumes (no GPU)."""
import numpy as np

from oracle import oracle as O
from paper_2605_12110_amd import synth

CAND = [8, 16, 32, 64, 128]


def _assign(curves, tau, cand=CAND):
    rec = np.asarray(curves, np.float64)[None]                       # one sample
    return O.assign_block_sizes(rec, cand, tau)[0].tolist()


def test_eq2_hand_cases():
    # head 0: recall falls slowly; head 1: falls off a cliff after 16; head 2: flat
    curves = [[0.98, 0.97, 0.965, 0.95, 0.90],
              [0.90, 0.89, 0.60, 0.40, 0.20],
              [0.50, 0.50, 0.50, 0.50, 0.50]]
    assert _assign(curves, 0.98) == [32, 16, 128]                     # thresholds 0.9604, 0.882, 0.49
    assert _assign(curves, 0.90) == [128, 16, 128]                    # 0.882, 0.81, 0.45
    assert _assign(curves, 0.20) == [128, 128, 128]
    assert _assign(curves, 1.0) == [8, 8, 128]                        # only ties with B_min pass


def test_eq2_smallest_candidate_always_qualifies_and_the_set_is_read_literally():
    assert _assign([[0.0, 0.0, 0.0, 0.0, 0.0]], 0.98) == [128]        # 0 >= tau * 0
    assert _assign([[0.7, 0.1, 0.1, 0.1, 0.1]], 0.98) == [8]
    # non-monotone curve: 64 passes although 32 fails; the maximum of the set is 64
    assert _assign([[0.80, 0.79, 0.50, 0.795, 0.60]], 0.98) == [64]
    # candidates need not be the default ladder
    assert _assign([[0.9, 0.9, 0.1]], 0.98, cand=[16, 64, 128]) == [64]


def test_eq2_uses_the_mean_over_calibration_samples():
    rng = np.random.default_rng(0)
    rec = rng.uniform(0.2, 1.0, size=(50, 6, 5))
    rec[:, :, 0] = np.maximum(rec[:, :, 0], 0.9)
    got, mean = O.assign_block_sizes(rec, CAND, 0.95)
    want_mean = rec.mean(axis=0)
    assert np.allclose(mean, want_mean, rtol=1e-14, atol=0)
    for h in range(6):
        ok = [k for k in range(5) if want_mean[h, k] >= 0.95 * want_mean[h, 0]]
        assert got[h] == CAND[max(ok)]
    # one sample far below the rest pulls a borderline head down: the rule sees means, not per-sample votes
    rec2 = np.full((4, 1, 2), 0.97)
    rec2[:, 0, 0] = 1.0
    assert O.assign_block_sizes(rec2, [8, 16], 0.96)[0].tolist() == [16]
    rec2[3, 0, 1] = 0.80
    assert O.assign_block_sizes(rec2, [8, 16], 0.96)[0].tolist() == [8]


def test_recall_is_the_selected_share_of_the_dense_softmax_mass_and_grows_to_one():
    wl = synth.make_workload(1, context=1024)
    st = O.build_centroids(wl)
    prev = None
    for T in (64, 256, 1024):
        wl.budget[:] = T
        r = O.decode_step(wl, st)
        rec = O.attention_recall(wl, r["sel_idx"], r["sel_cnt"])
        # identity used by the GPU path: recall = exp(lse over the selection - lse over the context)
        _, lse_sel = O.sparse_attention(wl, r["sel_idx"], r["sel_cnt"])
        _, lse_all = O.dense_attention(wl)
        assert np.allclose(rec, np.exp(lse_sel - lse_all), rtol=1e-12, atol=1e-15)
        assert np.all(rec > 0) and np.all(rec <= 1 + 1e-12)
        if prev is not None:
            assert np.all(rec >= prev - 1e-12)                        # holds on this input (not a law: selections need not nest)
        prev = rec
    assert np.allclose(prev, 1.0, rtol=0, atol=1e-12)                 # T >= L: everything selected
    hr = O.head_recall(wl, r["sel_idx"], r["sel_cnt"])
    assert hr.shape == (1, wl.num_kv_heads) and np.allclose(hr, 1.0)
