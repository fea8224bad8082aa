"""Pins for per-query-head selection (each query head of a grouped-query model selects by its own
score; the paper says "per head" and leaves the grouping open).  The oracle computes it as the method
applied to the model in which every query head is its own group (oracle.per_query_head_view); these
tests pin that construction to things it does not compute itself."""
import numpy as np

from oracle import oracle as O
from paper_2605_12110_amd import synth


def _wl(**kw):
    return synth.tiny_workload(seed=11, Bt=2, Hq=8, Hkv=2, P=16, seq_lens=(301, 512), block_size=(8, 32),
                               budget=(64, 96), **kw)


def test_view_repeats_each_kv_head_for_its_query_heads_and_leaves_queries_alone():
    wl = _wl()
    v = O.per_query_head_view(wl)
    G = wl.group
    assert v.num_kv_heads == wl.num_q_heads and v.group == 1
    assert v.block_size.tolist() == [8] * G + [32] * G
    for hq in range(wl.num_q_heads):
        for b in range(wl.batch):
            assert np.array_equal(v.key_rows(b, hq), wl.key_rows(b, hq // G))
            assert np.array_equal(v.value_rows(b, hq), wl.value_rows(b, hq // G))
    assert v.q is wl.q


def test_store_of_the_view_is_the_kv_heads_store_once_per_query_head():
    wl = _wl()
    st, sv = O.build_centroids(wl), O.build_centroids(O.per_query_head_view(wl))
    G = wl.group
    for b in range(wl.batch):
        for hq in range(wl.num_q_heads):
            s, t = b * wl.num_kv_heads + hq // G, b * wl.num_q_heads + hq
            assert np.array_equal(sv.codes[sv.off[t]:sv.off[t + 1]], st.codes[st.off[s]:st.off[s + 1]])
            assert np.array_equal(sv.qscale[t], st.qscale[s]) and np.array_equal(sv.qmin[t], st.qmin[s])


def test_a_head_selects_as_if_it_were_alone_in_the_model():
    """Query head hq's list and output are those of the default path on a model that holds only that
    query head and its KV head (an independent route: a different workload, sliced by hand)."""
    import copy
    wl = _wl()
    v = O.per_query_head_view(wl)
    ref = O.decode_step(v, O.build_centroids(v))
    G = wl.group
    for hq in (0, 3, 5):
        one = copy.copy(wl)
        one.num_q_heads = one.num_kv_heads = 1
        one.q = np.ascontiguousarray(wl.q[:, hq:hq + 1])
        one.k_cache = np.ascontiguousarray(wl.k_cache[:, hq // G:hq // G + 1])
        one.v_cache = np.ascontiguousarray(wl.v_cache[:, hq // G:hq // G + 1])
        one.block_size = wl.block_size[hq // G:hq // G + 1]
        r1 = O.decode_step(one, O.build_centroids(one))
        for b in range(wl.batch):
            t = b * wl.num_q_heads + hq
            k = r1["sel_cnt"][b]
            assert ref["sel_cnt"][t] == k
            assert np.array_equal(ref["sel_idx"][t, :k], r1["sel_idx"][b, :k])
            assert np.array_equal(ref["out"][b, hq], r1["out"][b, 0])


def test_identical_query_heads_select_what_their_group_selects():
    """If the G = 4 query heads of a group are equal, their sum is 4q: the same weights two binary
    places up, hence the same fixed-point image, the same ranking and the same selection as each head
    alone; the group path's output rows then equal the per-query-head rows."""
    wl = _wl()
    G = wl.group
    assert G == 4
    wl.q = np.repeat(wl.q[:, ::G], G, axis=1)
    grp = O.decode_step(wl, O.build_centroids(wl))
    v = O.per_query_head_view(wl)
    per = O.decode_step(v, O.build_centroids(v))
    for b in range(wl.batch):
        for hq in range(wl.num_q_heads):
            s, t = b * wl.num_kv_heads + hq // G, b * wl.num_q_heads + hq
            assert per["sel_cnt"][t] == grp["sel_cnt"][s]
            assert np.array_equal(per["sel_idx"][t, :per["sel_cnt"][t]], grp["sel_idx"][s, :grp["sel_cnt"][s]])
    assert np.array_equal(per["out"], grp["out"])


def test_budget_covering_the_context_makes_both_selections_dense():
    wl = _wl()
    wl.budget = np.array([4096, 4096], np.int32)
    v = O.per_query_head_view(wl)
    per = O.decode_step(v, O.build_centroids(v))
    dense, lse = O.dense_attention(wl)
    assert np.abs(per["out"] - dense).max() < 1e-12 and np.abs(per["lse"] - lse).max() < 1e-12


def test_own_selection_never_holds_less_of_a_heads_attention_than_the_groups():
    """The point of the variant: with unquantized exact scores a head's own Top-K maximises its own
    estimated mass; on inputs where heads of a group disagree, the head's attention recall under its
    own list is at least that under the group's list on average."""
    wl = synth.make_workload(1, context=2048, budget=256)
    grp = O.decode_step(wl, O.build_centroids(wl))
    v = O.per_query_head_view(wl)
    per = O.decode_step(v, O.build_centroids(v))
    G = wl.group
    rec_group = O.attention_recall(wl, grp["sel_idx"], grp["sel_cnt"])          # [Bt, Hq]
    rec_own = O.attention_recall(v, per["sel_idx"], per["sel_cnt"])
    assert rec_own.shape == rec_group.shape
    assert rec_own.mean() >= rec_group.mean() - 1e-9
