"""ctypes front end of the CPU oracle (absb_oracle.c).

TEST INFRASTRUCTURE ONLY: importable from tests/, from the smoke check and from the
benchmark's CPU-baseline leg, never from the product package.  It takes plain numpy
arrays (the ones the seeded generators produce) and returns numpy arrays.  No function
here contains arithmetic of the method: everything numeric happens in the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "absb_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_PREBUILT = os.environ.get("ABSB_ORACLE_LIB")      # another build of this file (the sanitizer build of tests/sanitized.py)

# -ffp-contract=off / no fast-math: every binary32 step is a single IEEE operation.
_CFLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
           "-fno-unsafe-math-optimizations", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (a checker being built is not the checker being used)."""
    if _PREBUILT and not force:
        return _PREBUILT
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", *_CFLAGS, _SRC, "-o", tmp, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_offsets.restype = C.c_int64
        _lib.orc_num_threads.restype = C.c_int
    return _lib


def _p(a: Optional[np.ndarray]):
    if a is None:
        return None
    assert a.flags["C_CONTIGUOUS"], "oracle arrays must be C-contiguous"
    return a.ctypes.data_as(C.c_void_p)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def num_threads() -> int:
    return int(lib().orc_num_threads())


def set_threads(n: int) -> None:
    lib().orc_set_threads(C.c_int(n))


MEAN, MINMAX = 0, 1         # block representation: mean pooling / channel-wise maxima and minima


@dataclass
class CentroidStore:
    """Widths below are for mean pooling; with max-min pooling every row is twice as wide
    (maxima first, then minima)."""
    off: np.ndarray        # int64 [nseg+1]
    cent: np.ndarray       # float32 [total, d]   (unquantized block representation)
    qscale: np.ndarray     # float32 [nseg, d]
    qmin: np.ndarray       # float32 [nseg, d]
    qinv: np.ndarray       # float32 [nseg, d]
    codes: np.ndarray      # uint8 [total, d/2]
    repr: int = MEAN


def _geom(wl):
    sp, sh, st = wl.strides
    return (C.c_int(wl.dtype), C.c_int(wl.batch), C.c_int(wl.num_q_heads), C.c_int(wl.num_kv_heads),
            C.c_int(wl.head_dim), C.c_int(wl.page_size), C.c_int64(sp), C.c_int64(sh), C.c_int64(st))


def offsets(wl) -> np.ndarray:
    nseg = wl.batch * wl.num_kv_heads
    off = np.zeros(nseg + 1, dtype=np.int64)
    lib().orc_offsets(C.c_int(wl.batch), C.c_int(wl.num_kv_heads), _p(_i32(wl.seq_lens)),
                      _p(_i32(wl.block_size)), _p(off))
    return off


def centroids(wl, off: np.ndarray) -> np.ndarray:
    dt, Bt, _, Hkv, d, P, sp, sh, st = _geom(wl)
    cent = np.empty((int(off[-1]), wl.head_dim), dtype=np.float32)
    pt = _i32(wl.page_table)
    lib().orc_centroids(dt, Bt, Hkv, d, P, sp, sh, st, _p(wl.k_cache), _p(pt), C.c_int(pt.shape[1]),
                        _p(_i32(wl.seq_lens)), _p(_i32(wl.block_size)), _p(off), _p(cent))
    return cent


def minmax_pool(wl, off: np.ndarray) -> np.ndarray:
    dt, Bt, _, Hkv, d, P, sp, sh, st = _geom(wl)
    rep = np.empty((int(off[-1]), 2 * wl.head_dim), dtype=np.float32)
    pt = _i32(wl.page_table)
    lib().orc_minmax_pool(dt, Bt, Hkv, d, P, sp, sh, st, _p(wl.k_cache), _p(pt), C.c_int(pt.shape[1]),
                          _p(_i32(wl.seq_lens)), _p(_i32(wl.block_size)), _p(off), _p(rep))
    return rep


def quant_params(off, cent):
    nseg, d = len(off) - 1, cent.shape[1]
    qscale = np.empty((nseg, d), np.float32)
    qmin = np.empty((nseg, d), np.float32)
    qinv = np.empty((nseg, d), np.float32)
    lib().orc_quant_params(C.c_int(nseg), C.c_int(d), _p(off), _p(cent), _p(qscale), _p(qmin), _p(qinv))
    return qscale, qmin, qinv


def quantize(off, cent, qmin, qinv) -> np.ndarray:
    nseg, d = len(off) - 1, cent.shape[1]
    cent = np.ascontiguousarray(cent, dtype=np.float32)
    codes = np.zeros((cent.shape[0], d // 2), np.uint8)
    lib().orc_quantize(C.c_int(nseg), C.c_int(d), _p(off), _p(cent), _p(qmin), _p(qinv), _p(codes))
    return codes


def dequantize(off, codes, qscale, qmin) -> np.ndarray:
    nseg, d = len(off) - 1, qscale.shape[1]
    out = np.empty((codes.shape[0], d), np.float32)
    lib().orc_dequantize(C.c_int(nseg), C.c_int(d), _p(off), _p(codes), _p(qscale), _p(qmin), _p(out))
    return out


def build_centroids(wl, repr: int = MEAN) -> CentroidStore:
    """O1-O3: block representation (means, or maxima and minima), per-channel ranges, INT4 codes."""
    off = offsets(wl)
    cent = centroids(wl, off) if repr == MEAN else minmax_pool(wl, off)
    qscale, qmin, qinv = quant_params(off, cent)
    codes = quantize(off, cent, qmin, qinv)
    return CentroidStore(off, cent, qscale, qmin, qinv, codes, repr)


def quantize_variant(off, cent, bits: int, symmetric: bool):
    """Sec. 3.3 design space: (qscale, qmin, codes one per byte, stored code of zero)."""
    nseg, d = len(off) - 1, cent.shape[1]
    cent = np.ascontiguousarray(cent, dtype=np.float32)
    qscale = np.empty((nseg, d), np.float32)
    qmin = np.empty((nseg, d), np.float32)
    codes = np.zeros((cent.shape[0], d), np.uint8)
    lib().orc_quantize_variant(C.c_int(nseg), C.c_int(d), _p(off), _p(cent), C.c_int(bits), C.c_int(int(symmetric)),
                               _p(qscale), _p(qmin), _p(codes))
    return qscale, qmin, codes, ((1 << (bits - 1)) - 1 if symmetric else 0)


def score_variant(wl, off, codes, qscale, zero: int):
    nseg = wl.batch * wl.num_kv_heads
    scores = np.empty(int(off[-1]), np.int32)
    ex = np.empty(nseg, np.int32)
    lib().orc_score_variant(C.c_int(wl.dtype), C.c_int(wl.batch), C.c_int(wl.num_q_heads), C.c_int(wl.num_kv_heads),
                            C.c_int(wl.head_dim), _p(np.ascontiguousarray(wl.q)), _p(codes), _p(qscale), C.c_int(zero),
                            _p(off), _p(scores), _p(ex))
    return scores, ex


def tail_state(wl, repr: int = MEAN) -> np.ndarray:
    """Pooled state of every segment's last block (running sum, or running maxima and minima)."""
    dt, Bt, _, Hkv, d, P, sp, sh, st = _geom(wl)
    nseg = wl.batch * wl.num_kv_heads
    tail = np.zeros((nseg, wl.head_dim * (repr + 1)), np.float32)
    pt = _i32(wl.page_table)
    lib().orc_tail_state(dt, C.c_int(repr), Bt, Hkv, d, P, sp, sh, st, _p(wl.k_cache), _p(pt), C.c_int(pt.shape[1]),
                         _p(_i32(wl.seq_lens)), _p(_i32(wl.block_size)), _p(tail))
    return tail


def append_token(wl, store: CentroidStore, tail: np.ndarray, clamped: Optional[np.ndarray] = None):
    """The token at position L_b - 1 of every request (wl.seq_lens already counts it, the key is in
    wl.k_cache) joins the store under its frozen ranges.  Returns (new store in the tight layout of
    the new lengths, block values [nseg, W]); `tail` is updated in place, and so is `clamped`
    (int32 [nseg], optional): per segment the running count of values in completed blocks that the
    frozen ranges did not hold."""
    dt, Bt, _, Hkv, d, P, sp, sh, st = _geom(wl)
    nseg = wl.batch * wl.num_kv_heads
    W = wl.head_dim * (store.repr + 1)
    rows = np.zeros((nseg, W // 2), np.uint8)
    values = np.empty((nseg, W), np.float32)
    pt = _i32(wl.page_table)
    lib().orc_append_token(dt, C.c_int(store.repr), Bt, Hkv, d, P, sp, sh, st, _p(wl.k_cache), _p(pt),
                           C.c_int(pt.shape[1]), _p(_i32(wl.seq_lens)), _p(_i32(wl.block_size)), _p(store.qscale),
                           _p(store.qmin), _p(tail), _p(rows), _p(values), _p(clamped))
    new_off = offsets(wl)
    codes = np.zeros((int(new_off[-1]), W // 2), np.uint8)
    cent = None if store.cent is None else np.zeros((int(new_off[-1]), W), np.float32)
    for s in range(nseg):
        n_old = int(store.off[s + 1] - store.off[s])
        n_new = int(new_off[s + 1] - new_off[s])
        assert n_new in (n_old, n_old + 1)
        keep = n_new - 1                               # rows of closed blocks carry over unchanged
        codes[new_off[s]:new_off[s] + keep] = store.codes[store.off[s]:store.off[s] + keep]
        codes[new_off[s] + keep] = rows[s]
        if cent is not None:
            cent[new_off[s]:new_off[s] + keep] = store.cent[store.off[s]:store.off[s] + keep]
            cent[new_off[s] + keep] = values[s]
    return CentroidStore(new_off, cent, store.qscale, store.qmin, store.qinv, codes, store.repr), values


def score(wl, store: CentroidStore, q: Optional[np.ndarray] = None, want_weights: bool = False):
    """O4: int32 fixed-point scores for every centroid, per-segment exponent."""
    q = wl.q if q is None else q
    nseg = wl.batch * wl.num_kv_heads
    scores = np.empty(int(store.off[-1]), np.int32)
    ex = np.empty(nseg, np.int32)
    width = wl.head_dim * (2 if store.repr == MINMAX else 1)
    wq = np.empty((nseg, width), np.int32) if want_weights else None
    fn = lib().orc_score_minmax if store.repr == MINMAX else lib().orc_score
    fn(C.c_int(wl.dtype), C.c_int(wl.batch), C.c_int(wl.num_q_heads), C.c_int(wl.num_kv_heads),
       C.c_int(wl.head_dim), _p(np.ascontiguousarray(q)), _p(store.codes), _p(store.qscale),
       _p(store.off), _p(scores), _p(ex), _p(wq))
    return (scores, ex, wq) if want_weights else (scores, ex)


def score_groupmax(wl, store: CentroidStore, q: Optional[np.ndarray] = None, want_weights: bool = False):
    """Group score = maximum over the group's query heads of q_g . c^_j, on one fixed-point scale per
    group (mean pooling only).  Returns (scores, exponents[, wq [nseg, G, d], zq [nseg, G]])."""
    assert store.repr == MEAN
    q = wl.q if q is None else q
    nseg = wl.batch * wl.num_kv_heads
    scores = np.empty(int(store.off[-1]), np.int32)
    ex = np.empty(nseg, np.int32)
    wq = np.empty((nseg, wl.group, wl.head_dim), np.int32) if want_weights else None
    zq = np.empty((nseg, wl.group), np.int32) if want_weights else None
    lib().orc_score_groupmax(C.c_int(wl.dtype), C.c_int(wl.batch), C.c_int(wl.num_q_heads), C.c_int(wl.num_kv_heads),
                             C.c_int(wl.head_dim), _p(np.ascontiguousarray(q)), _p(store.codes), _p(store.qscale),
                             _p(store.qmin), _p(store.off), _p(scores), _p(ex), _p(wq), _p(zq))
    return (scores, ex, wq, zq) if want_weights else (scores, ex)


def topk_raw(Bt, Hkv, off, block_size, budget, scores, sel_stride, seq_lens=None, sink_tokens=0, recent_tokens=0):
    nseg = Bt * Hkv
    sel_idx = np.empty((nseg, sel_stride), np.int32)
    sel_cnt = np.empty(nseg, np.int32)
    lens = None if seq_lens is None else _i32(seq_lens)
    lib().orc_topk(C.c_int(Bt), C.c_int(Hkv), _p(np.ascontiguousarray(off, dtype=np.int64)), _p(_i32(block_size)),
                   _p(_i32(budget)), _p(_i32(scores)), _p(sel_idx), _p(sel_cnt), C.c_int(sel_stride),
                   _p(lens), C.c_int(sink_tokens), C.c_int(recent_tokens))
    return sel_idx, sel_cnt


def topk(wl, off, scores, sel_stride: Optional[int] = None, budget=None, sink_tokens=0, recent_tokens=0):
    """O5: per segment the K_s best blocks (score desc, index asc), emitted ascending, -1 padded.
    Blocks holding the first `sink_tokens` / last `recent_tokens` tokens rank first (forced)."""
    budget = wl.budget if budget is None else budget
    if sel_stride is None:
        # widest possible list: every block of the longest segment (always enough)
        sel_stride = int(np.max(np.diff(off))) if len(off) > 1 else 1
        sel_stride = max(sel_stride, 1)
    return topk_raw(wl.batch, wl.num_kv_heads, off, wl.block_size, budget, scores, sel_stride, wl.seq_lens,
                    sink_tokens, recent_tokens)


def sparse_attention(wl, sel_idx, sel_cnt, sm_scale: Optional[float] = None, q=None):
    """O6: fp64 attention over the selected blocks.  Returns (out [Bt,Hq,d], lse [Bt,Hq])."""
    q = wl.q if q is None else q
    sm = float(1.0 / np.sqrt(wl.head_dim)) if sm_scale is None else float(sm_scale)
    out = np.empty((wl.batch, wl.num_q_heads, wl.head_dim), np.float64)
    lse = np.empty((wl.batch, wl.num_q_heads), np.float64)
    sel_idx = _i32(sel_idx)
    pt = _i32(wl.page_table)
    lib().orc_sparse_attention(*_geom(wl), _p(np.ascontiguousarray(q)), _p(wl.k_cache), _p(wl.v_cache), _p(pt),
                               C.c_int(pt.shape[1]), _p(_i32(wl.seq_lens)), _p(_i32(wl.block_size)),
                               _p(sel_idx), _p(_i32(sel_cnt)), C.c_int(sel_idx.shape[1]), C.c_double(sm),
                               _p(out), _p(lse))
    return out, lse


def dense_attention(wl, sm_scale: Optional[float] = None, q=None):
    """Eq. (1) over the whole context, fp64."""
    q = wl.q if q is None else q
    sm = float(1.0 / np.sqrt(wl.head_dim)) if sm_scale is None else float(sm_scale)
    out = np.empty((wl.batch, wl.num_q_heads, wl.head_dim), np.float64)
    lse = np.empty((wl.batch, wl.num_q_heads), np.float64)
    pt = _i32(wl.page_table)
    lib().orc_dense_attention(*_geom(wl), _p(np.ascontiguousarray(q)), _p(wl.k_cache), _p(wl.v_cache), _p(pt),
                              C.c_int(pt.shape[1]), _p(_i32(wl.seq_lens)), C.c_double(sm), _p(out), _p(lse))
    return out, lse


def attention_recall(wl, sel_idx, sel_cnt, sm_scale: Optional[float] = None):
    """Share of the dense softmax mass on the selected tokens (Sec. 2.3), per query head."""
    sm = float(1.0 / np.sqrt(wl.head_dim)) if sm_scale is None else float(sm_scale)
    rec = np.empty((wl.batch, wl.num_q_heads), np.float64)
    sel_idx = _i32(sel_idx)
    pt = _i32(wl.page_table)
    lib().orc_attention_recall(*_geom(wl), _p(wl.q), _p(wl.k_cache), _p(pt), C.c_int(pt.shape[1]),
                               _p(_i32(wl.seq_lens)), _p(_i32(wl.block_size)), _p(sel_idx), _p(_i32(sel_cnt)),
                               C.c_int(sel_idx.shape[1]), C.c_double(sm), _p(rec))
    return rec


def head_recall(wl, sel_idx, sel_cnt, sm_scale: Optional[float] = None) -> np.ndarray:
    """Attention recall per (request, KV head): the mean over the group's query heads."""
    rec = attention_recall(wl, sel_idx, sel_cnt, sm_scale)
    return rec.reshape(wl.batch, wl.num_kv_heads, wl.group).mean(axis=2)


def assign_block_sizes(recall, candidates, tau: float):
    """Eq. (2).  recall [n_samples, n_heads, n_candidates] -> (block size per head, mean recall [heads, cands])."""
    recall = np.ascontiguousarray(recall, dtype=np.float64)
    n, nh, nB = recall.shape
    cand = _i32(candidates)
    assert len(cand) == nB and np.all(np.diff(cand) > 0)
    out = np.empty(nh, np.int32)
    mean = np.empty((nh, nB), np.float64)
    lib().orc_assign_block_sizes(C.c_int(n), C.c_int(nh), C.c_int(nB), _p(recall), _p(cand), C.c_double(tau),
                                 _p(out), _p(mean))
    return out, mean


def planted_recall(wl, sel_idx, sel_cnt) -> float:
    """Fraction of the generator's planted heavy tokens whose block was selected (diagnostic)."""
    hit = tot = 0
    for (b, h), pos in wl.planted.items():
        s = b * wl.num_kv_heads + h
        chosen = set(int(x) for x in sel_idx[s, :sel_cnt[s]])
        blocks = pos // int(wl.block_size[h])
        hit += sum(1 for j in blocks if int(j) in chosen)
        tot += len(blocks)
    return hit / max(tot, 1)


def decode_step(wl, store: CentroidStore, sel_stride: Optional[int] = None, sink_tokens=0, recent_tokens=0,
                group_max: bool = False):
    """O4 -> O5 -> O6 given a prebuilt centroid store: the per-step hot path.  `group_max`: the group's
    shared score is the maximum over its query heads instead of their sum."""
    scores, ex = score_groupmax(wl, store) if group_max else score(wl, store)
    sel_idx, sel_cnt = topk(wl, store.off, scores, sel_stride, sink_tokens=sink_tokens, recent_tokens=recent_tokens)
    out, lse = sparse_attention(wl, sel_idx, sel_cnt)
    return dict(scores=scores, score_exp=ex, sel_idx=sel_idx, sel_cnt=sel_cnt, out=out, lse=lse)


def per_query_head_view(wl, caches: bool = True):
    """Per-query-head selection (every query head ranks and selects blocks by its own score and attends
    over its own list) is, by definition, the method applied to a model in which every query head is a
    group of its own: Hq KV heads, KV head hq holding the keys and values of the original KV head
    hq // G, with that head's block size.  This returns that model as a workload (the caches with
    their heads repeated G times): the oracle's functions applied to it ARE the per-query-head path,
    and a store built from it holds, for every query head, a copy of its KV head's store segment.
    Heavy-token bookkeeping is carried over per query head.  `caches=False` leaves the caches out (for
    diagnostics that need the head bookkeeping only)."""
    import copy
    G = wl.group
    v = copy.copy(wl)
    v.num_kv_heads = wl.num_q_heads
    v.block_size = np.repeat(np.asarray(wl.block_size, np.int32), G)
    v.k_cache = np.repeat(wl.k_cache, G, axis=1) if caches else None
    v.v_cache = np.repeat(wl.v_cache, G, axis=1) if caches else None
    v.planted = {(b, h * G + g): pos for (b, h), pos in wl.planted.items() for g in range(G)}
    return v
