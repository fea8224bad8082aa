"""Device-side holder for a synthetic workload: uploads the generator's arrays to HBM with
torch (memory and streams only) and wires them into the binding's Layer/Batch records."""
from __future__ import annotations

from typing import Optional

import numpy as np
import torch

from . import absb


def _up(a: np.ndarray, dtype=None, device="cuda:0"):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.view(dtype)
    return t.to(device)


class DeviceWorkload:
    """Everything one layer's decode step needs, resident on the GPU."""

    def __init__(self, wl, device: str = "cuda:0", budget: Optional[np.ndarray] = None,
                 block_repr: int = absb.REPR_MEAN, block_size: Optional[np.ndarray] = None,
                 share: Optional["DeviceWorkload"] = None, sink_tokens: int = 0, recent_tokens: int = 0,
                 cap_lens: Optional[np.ndarray] = None, selection: int = absb.SELECT_GROUP,
                 opts: Optional[dict] = None):
        """`block_size` / `budget` override the workload's; `share` reuses another holder's resident
        caches, queries, lengths and page table (same workload under other block sizes or budgets);
        `cap_lens` lays the store out for contexts that grow up to those lengths (set_lens/append);
        `opts`: fields of absb_launch_opts that shape buffers (split_tokens, unit_tokens, ...)."""
        self.wl = wl
        self.device = device
        tdt = torch.float16 if wl.dtype == absb.F16 else torch.bfloat16
        self.torch_dtype = tdt
        budget = wl.budget if budget is None else np.asarray(budget, dtype=np.int32)
        self.block_size = np.asarray(wl.block_size if block_size is None else block_size, dtype=np.int32)
        self.layer = absb.Layer(wl.num_q_heads, wl.num_kv_heads, wl.head_dim, wl.page_size, wl.dtype,
                                self.block_size, wl.strides, block_repr=block_repr, sink_tokens=sink_tokens,
                                recent_tokens=recent_tokens, selection=selection)
        width = wl.head_dim * (2 if block_repr == absb.REPR_MINMAX else 1)      # values per block
        if share is None:
            self.k_cache = _up(wl.k_cache.view(np.int16), tdt, device)
            self.v_cache = _up(wl.v_cache.view(np.int16), tdt, device)
            self.q = _up(wl.q.view(np.int16), tdt, device)
            self.seq_lens = _up(wl.seq_lens.astype(np.int32), None, device)
            self.page_table = _up(wl.page_table.astype(np.int32), None, device)
        else:
            assert share.wl is wl
            self.k_cache, self.v_cache, self.q = share.k_cache, share.v_cache, share.q
            self.seq_lens, self.page_table = share.seq_lens, share.page_table
        self.budget = _up(budget.astype(np.int32), None, device)
        self.batch = absb.Batch(seq_lens_host=wl.seq_lens, budget_host=budget, seq_lens=self.seq_lens,
                                page_table=self.page_table, budget=self.budget, opts=absb.LaunchOpts(**(opts or {})))
        if cap_lens is not None:
            # buffers are sized for the longest contexts; the layout (offsets) stays that of cap_lens
            cap = np.asarray(cap_lens, dtype=np.int32)
            self.batch.cap_lens_host = cap
            self.batch.seq_lens_host = cap
            self.plan = absb.absb_plan(self.layer, self.batch)
            self.batch.seq_lens_host = wl.seq_lens
        else:
            self.plan = absb.absb_plan(self.layer, self.batch)
        self.cent_off = _up(self.plan.cent_off, None, device)
        self.batch.cent_off = self.cent_off
        nseg = wl.batch * wl.num_kv_heads          # store segments
        self.nseg = nseg
        per_q = selection == absb.SELECT_PER_QUERY_HEAD
        nsel = wl.batch * (wl.num_q_heads if per_q else wl.num_kv_heads)      # selection segments
        self.nsel = nsel
        rk = wl.num_q_heads // wl.num_kv_heads if per_q else 1
        total = self.plan.total_centroids
        self.codes = torch.empty((total, width // 2), dtype=torch.uint8, device=device)
        self.qscale = torch.empty((nseg, width), dtype=torch.float32, device=device)
        self.qmin = torch.empty((nseg, width), dtype=torch.float32, device=device)
        self.batch.qmin = self.qmin
        self.scores = torch.empty((total * rk,), dtype=torch.int32, device=device)
        self.score_exp = torch.empty((nsel,), dtype=torch.int32, device=device)
        self.sel_stride = max(self.plan.sel_stride, 1)
        self._sel_buf = torch.empty((nsel * self.sel_stride,), dtype=torch.int32, device=device)
        self.sel_idx = self._sel_buf.view(nsel, self.sel_stride)
        self.sel_cnt = torch.empty((nsel,), dtype=torch.int32, device=device)
        self.out = torch.empty((wl.batch, wl.num_q_heads, wl.head_dim), dtype=tdt, device=device)
        self.lse = torch.empty((wl.batch, wl.num_q_heads), dtype=torch.float32, device=device)
        self.tail = torch.empty((nseg, width), dtype=torch.float32, device=device)
        self.clamped = torch.zeros((nseg,), dtype=torch.int32, device=device)   # values outside the frozen ranges
        self.workspace = torch.empty((self.plan.workspace_bytes + 256,), dtype=torch.uint8, device=device)
        self.scribble(0xA5)
        if cap_lens is not None:
            self.set_lens(wl.seq_lens)             # the lists are as wide as the current lengths make them

    def clone(self) -> "DeviceWorkload":
        """A second resident copy of everything a step reads or writes, at other addresses: same
        workload, same block sizes and budgets, the centroid store copied as it stands.  Stepping
        through several clones in turn keeps a benchmark from re-reading lines that an earlier step left
        in a cache."""
        c = DeviceWorkload.__new__(DeviceWorkload)
        c.__dict__.update(self.__dict__)
        for name in ("k_cache", "v_cache", "q", "seq_lens", "page_table", "budget", "cent_off", "codes", "qscale", "qmin",
                     "scores", "score_exp", "_sel_buf", "sel_cnt", "out", "lse", "tail", "clamped", "workspace"):
            setattr(c, name, getattr(self, name).clone())
        c.sel_idx = c._sel_buf[:c.nsel * c.sel_stride].view(c.nsel, c.sel_stride)
        c.batch = absb.Batch(seq_lens_host=self.batch.seq_lens_host, budget_host=self.batch.budget_host,
                             seq_lens=c.seq_lens, page_table=c.page_table, cent_off=c.cent_off, budget=c.budget,
                             cap_lens_host=self.batch.cap_lens_host, qmin=c.qmin,
                             opts=absb.LaunchOpts(**vars(self.batch.opts)))
        absb.absb_workspace_init(c.layer, c.batch, c.workspace)
        return c

    def scribble(self, value: int, stream=None):
        """Poison the workspace (no entry point may depend on its previous contents), then clear its
        counters the way a caller must before the first fused step on a fresh workspace."""
        self.workspace.fill_(value)
        absb.absb_workspace_init(self.layer, self.batch, self.workspace, stream)

    # -- entry points, in path order
    def build(self, stream=None):
        absb.absb_build_centroids(self.layer, self.batch, self.k_cache, self.codes, self.qscale, self.qmin,
                                  self.workspace, stream)

    # -- growing contexts
    def set_lens(self, lens):
        """New context lengths (within cap_lens); the keys of the new tokens are already in the cache."""
        lens = np.asarray(lens, dtype=np.int32)
        self.seq_lens.copy_(torch.from_numpy(lens))
        self.batch.seq_lens_host = lens
        # the list width follows the lengths (budgets beyond a context select all of its blocks):
        # the lists of the current lengths are [segments][sel_stride] at the start of the buffer
        self.sel_stride = max(absb.absb_plan(self.layer, self.batch).sel_stride, 1)
        self.sel_idx = self._sel_buf[:self.nsel * self.sel_stride].view(self.nsel, self.sel_stride)

    def tail_init(self, stream=None):
        absb.absb_tail_init(self.layer, self.batch, self.k_cache, self.tail, stream)

    def append_token(self, stream=None):
        absb.absb_append_token(self.layer, self.batch, self.k_cache, self.codes, self.qscale, self.qmin,
                               self.tail, self.clamped, stream)

    def load_store(self, codes: np.ndarray, qscale: np.ndarray, qmin: np.ndarray):
        """Install a centroid store computed elsewhere (e.g. by the oracle, for stage-isolated tests)."""
        self.codes.copy_(torch.from_numpy(np.ascontiguousarray(codes)))
        self.qscale.copy_(torch.from_numpy(np.ascontiguousarray(qscale)))
        self.qmin.copy_(torch.from_numpy(np.ascontiguousarray(qmin)))

    def score(self, stream=None):
        absb.absb_score(self.layer, self.batch, self.q, self.codes, self.qscale, self.scores, self.score_exp, stream)

    def topk(self, stream=None):
        absb.absb_topk(self.layer, self.batch, self.scores, self.sel_idx, self.sel_cnt, self.sel_stride,
                       None, stream)

    def sparse_decode(self, stream=None):
        absb.absb_sparse_decode(self.layer, self.batch, self.q, self.k_cache, self.v_cache, self.sel_idx,
                                self.sel_cnt, self.sel_stride, self.out, self.lse, self.workspace, stream)

    def decode_fused(self, stream=None, want_sel: bool = True):
        absb.absb_decode_fused(self.layer, self.batch, self.q, self.codes, self.qscale, self.k_cache,
                               self.v_cache, self.out, self.lse, self.sel_idx if want_sel else None,
                               self.sel_cnt if want_sel else None, self.workspace, stream)

    def status(self) -> int:
        """The one-launch step's status word (0 = no wait ran out); synchronises."""
        off = absb.absb_status_offset(self.layer, self.batch)
        return int(self.workspace[off:off + 4].view(torch.int32).item())

    def check_device_contents(self, lists: bool = False) -> None:
        """Debug aid: the library trusts what device arrays hold (a page index out of range is undefined
        behaviour there).  This copies the index arrays back and checks them on the host: lengths and
        budgets equal to their host twins, offsets equal to the plan's, every page-table entry a context
        reaches inside the caches, and (`lists`) every list well formed: counts within the list width,
        indices ascending and inside their segments, -1 behind them.  Raises AssertionError naming the
        first violation.  Synchronises; not for timed code."""
        wl = self.wl
        lens = np.asarray(self.batch.seq_lens_host, dtype=np.int64)
        assert np.array_equal(self.seq_lens.cpu().numpy(), lens), "seq_lens differs from seq_lens_host"
        assert np.array_equal(self.budget.cpu().numpy(), np.asarray(self.batch.budget_host)), "budget differs from budget_host"
        assert np.array_equal(self.cent_off.cpu().numpy(), self.plan.cent_off), "cent_off differs from absb_plan's"
        pt = self.page_table.cpu().numpy()
        npages = int(self.k_cache.shape[0])
        for b, L in enumerate(lens):
            used = pt[b, :-(-int(L) // wl.page_size)]
            assert used.size == 0 or (used.min() >= 0 and used.max() < npages), f"page table of request {b} leaves the cache"
        if lists:
            cnt, idx = self.sel_cnt.cpu().numpy(), self.sel_idx.cpu().numpy()
            rk = self.nsel // self.nseg
            for t in range(self.nsel):
                s = (t // (wl.num_kv_heads * rk)) * wl.num_kv_heads + (t % (wl.num_kv_heads * rk)) // rk
                b, h = divmod(s, wl.num_kv_heads)
                n = -(-int(lens[b]) // int(self.block_size[h]))
                k = int(cnt[t])
                assert 0 <= k <= min(n, self.sel_stride), f"sel_cnt[{t}] = {k}"
                row = idx[t, :k]
                assert k == 0 or (row.min() >= 0 and row.max() < n and np.all(np.diff(row) > 0)), f"sel_idx[{t}] malformed"
                assert np.all(idx[t, k:] == -1), f"sel_idx[{t}] not padded"

    # -- results back on the host
    def out_f32(self) -> np.ndarray:
        return self.out.float().cpu().numpy()
