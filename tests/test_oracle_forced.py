"""Pins for the oracle's forced-block selection policy (no GPU): blocks that hold one of the first
`sink_tokens` or last `recent_tokens` tokens always rank first; the rest of K_s is the plain Top-K
(Sec. 3.4, kernel 2) of the other blocks.  Checked against an independent numpy construction."""
import itertools

import numpy as np

from oracle import oracle as O


def _select(scores, B, T, L, sink, recent, stride=None):
    scores = np.asarray(scores, np.int32)
    N = len(scores)
    assert N == -(-L // B)
    off = np.array([0, N], np.int64)
    stride = max(N, 1) if stride is None else stride
    idx, cnt = O.topk_raw(1, 1, off, [B], [T], scores, stride, [L], sink, recent)
    return idx[0, :cnt[0]].tolist(), int(cnt[0])


def _reference(scores, B, T, L, sink, recent):
    """Forced set by token arithmetic, then lexsort of the others: written without the score trick."""
    N = len(scores)
    K = min(N, -(-T // B))
    forced = [j for j in range(N)
              if any(t < sink or t >= L - recent for t in range(j * B, min((j + 1) * B, L)))]
    if len(forced) >= K:
        return sorted(forced[:K])                      # lowest indices first: sinks before recents
    rest = [j for j in range(N) if j not in forced]
    order = sorted(rest, key=lambda j: (-int(scores[j]), j))
    return sorted(forced + order[:K - len(forced)])


def test_forced_blocks_hand_cases():
    # 10 blocks of 8 tokens, L = 77 (last block holds 5 tokens); scores favour the middle
    sc = [0, 1, 2, 9, 8, 7, 3, 2, 1, 0]
    assert _select(sc, 8, 24, 77, 0, 0)[0] == [3, 4, 5]
    assert _select(sc, 8, 24, 77, 1, 0)[0] == [0, 3, 4]                 # one sink token forces block 0
    assert _select(sc, 8, 24, 77, 9, 0)[0] == [0, 1, 3]                 # nine sink tokens reach into block 1
    assert _select(sc, 8, 24, 77, 0, 5)[0] == [3, 4, 9]                 # the last 5 tokens are exactly block 9
    assert _select(sc, 8, 24, 77, 0, 6)[0] == [3, 8, 9]                 # a sixth reaches back into block 8
    assert _select(sc, 8, 24, 77, 8, 5)[0] == [0, 3, 9]
    assert _select(sc, 8, 16, 77, 16, 13)[0] == [0, 1]                  # more forced blocks than K: lowest indices
    assert _select(sc, 8, 800, 77, 3, 3)[0] == list(range(10))          # K = N: everything


def test_forced_blocks_match_the_token_level_construction_exhaustively():
    rng = np.random.default_rng(11)
    for B, L in ((8, 61), (16, 100), (8, 8), (32, 33)):
        N = -(-L // B)
        for sink, recent in itertools.product((0, 1, B, B + 1, 3 * B), (0, 1, L % B or B, B + 2, L)):
            for T in (1, B, 3 * B, L):
                sc = rng.integers(-5, 6, size=N)                         # many ties
                got, cnt = _select(sc, B, T, L, sink, recent)
                want = _reference(sc, B, T, L, sink, recent)
                assert got == want, (B, L, sink, recent, T, sc.tolist())
                assert cnt == min(N, -(-T // B))


def test_forced_block_outranks_every_score_even_the_largest_integer():
    big = 2 ** 31 - 1
    assert _select([big, big, 0, 0], 8, 8, 32, 0, 1)[0] == [3]
    assert _select([big, big, 0, -2 ** 31], 8, 16, 32, 0, 1)[0] == [0, 3]


def test_no_forcing_is_the_plain_selection():
    rng = np.random.default_rng(12)
    sc = rng.integers(-100, 100, size=37)
    off = np.array([0, 37], np.int64)
    a = O.topk_raw(1, 1, off, [8], [64], sc, 37)
    b = O.topk_raw(1, 1, off, [8], [64], sc, 37, [37 * 8], 0, 0)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
