"""Design-space study of Sec. 3.3 on synthetic inputs, on the CPU oracle only: Top-K recall of the
block selection under 2/4/8-bit, symmetric/asymmetric per-channel centroid quantization, against
the selection made with the unquantized centroids.  Prints a markdown table.

    python -m oracle.quant_ablation
"""
import numpy as np

from oracle import oracle as O
from paper_2605_12110_amd import synth

CASES = [("config 1 (4K, planted keys)", dict(config=1)),
         ("config 2 (low-rank keys, 2 x 32K)", dict(config=2, batch=2)),
         ("config 3 (Zipf heavy tokens, 64K)", dict(config=3, context=65536, budget=2048))]


def recall_table(wl):
    st = O.build_centroids(wl)
    q = synth.bits_to_f32(wl.q, wl.dtype).astype(np.float64)
    G, Hkv = wl.group, wl.num_kv_heads
    exact = np.empty(int(st.off[-1]))
    for s in range(wl.batch * Hkv):
        b, h = divmod(s, Hkv)
        u = q[b, h * G:(h + 1) * G].sum(axis=0)
        exact[st.off[s]:st.off[s + 1]] = st.cent[st.off[s]:st.off[s + 1]].astype(np.float64) @ u
    # order-preserving integer image of the exact scores (per segment), then the same selection rule
    key = np.empty(len(exact), np.int32)
    for s in range(wl.batch * Hkv):
        seg = exact[st.off[s]:st.off[s + 1]]
        order = np.argsort(np.argsort(seg, kind="stable"), kind="stable")
        key[st.off[s]:st.off[s + 1]] = order.astype(np.int32)
    ref_idx, ref_cnt = O.topk(wl, st.off, key)
    out = {}
    for bits in (2, 4, 8):
        for sym in (True, False):
            qs, qm, codes, zero = O.quantize_variant(st.off, st.cent, bits, sym)
            sc, _ = O.score_variant(wl, st.off, codes, qs, zero)
            idx, cnt = O.topk(wl, st.off, sc)
            hits = sum(len(set(idx[s, :cnt[s]].tolist()) & set(ref_idx[s, :ref_cnt[s]].tolist()))
                       for s in range(wl.batch * Hkv))
            out[(bits, sym)] = hits / max(int(ref_cnt.sum()), 1)
    return out


def main():
    cols = [(2, True), (2, False), (4, True), (4, False), (8, True), (8, False)]
    print("| workload | " + " | ".join(f"INT{b} {'sym' if s else 'asym'}" for b, s in cols) + " |")
    print("|---|" + "---|" * len(cols))
    for name, kw in CASES:
        kw = dict(kw)
        wl = synth.make_workload(kw.pop("config"), **kw)
        r = recall_table(wl)
        print(f"| {name} | " + " | ".join(f"{r[c]:.3f}" for c in cols) + " |", flush=True)


if __name__ == "__main__":
    main()
