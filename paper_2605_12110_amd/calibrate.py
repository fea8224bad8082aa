"""Offline calibration of the per-head block sizes (Sec. 3.2): for every calibration sample and
every candidate block size, run the decode path with that size on all heads, measure the
attention recall of its selection (Sec. 2.3), and apply Eq. (2) to the means.

Everything numeric happens in libabsb: the store build, score, selection and attention kernels
produce the two log-sum-exp arrays, absb_head_recall turns them into recall per (request, KV head),
absb_assign_block_sizes takes the mean over the samples and applies Eq. (2).  This module only loops
and moves buffers.
"""
from __future__ import annotations

from typing import Iterable, Sequence

import numpy as np
import torch

from . import absb
from .device import DeviceWorkload

DEFAULT_CANDIDATES = (8, 16, 32, 64, 128)


def measure_recall(wl, candidates: Sequence[int] = DEFAULT_CANDIDATES, budget=None,
                   block_repr: int = absb.REPR_MEAN, device: str = "cuda:0") -> np.ndarray:
    """Recall(h, B) of one calibration input, one row per request: float32 [Bt, Hkv, len(candidates)]
    (every request is a sample of Eq. (2); the mean over samples is taken by absb_assign_block_sizes)."""
    Hkv = wl.num_kv_heads
    budget = wl.budget if budget is None else np.broadcast_to(np.asarray(budget, np.int32), (wl.batch,))
    # dense pass: a budget that covers the context selects every block, whatever the block size
    dense = DeviceWorkload(wl, device, budget=wl.seq_lens, block_repr=block_repr,
                           block_size=np.full(Hkv, candidates[0], np.int32))
    dense.build()
    dense.decode_fused(want_sel=False)
    out = np.empty((wl.batch, Hkv, len(candidates)), np.float32)
    recall = torch.empty((wl.batch * Hkv,), dtype=torch.float32, device=device)
    for k, B in enumerate(candidates):
        dw = DeviceWorkload(wl, device, budget=budget, block_repr=block_repr,
                            block_size=np.full(Hkv, B, np.int32), share=dense)
        dw.build()
        dw.decode_fused(want_sel=False)
        absb.absb_head_recall(dw.layer, dw.batch, dw.lse, dense.lse, recall)
        out[:, :, k] = recall.cpu().numpy().reshape(wl.batch, Hkv)
        del dw
    return out


def calibrate(samples: Iterable, candidates: Sequence[int] = DEFAULT_CANDIDATES, tau: float = 0.98, budget=None,
              block_repr: int = absb.REPR_MEAN, device: str = "cuda:0"):
    """Eq. (2) over calibration samples (workloads of one layer shape).
    Returns (block size per KV head, mean recall [Hkv, candidates], per-sample recall [n, Hkv, candidates])."""
    per_sample = np.concatenate([measure_recall(wl, candidates, budget, block_repr, device) for wl in samples])
    sizes, mean = absb.absb_assign_block_sizes(per_sample, candidates, tau)
    return sizes, mean, per_sample
