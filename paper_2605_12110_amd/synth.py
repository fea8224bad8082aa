"""Seeded synthetic decode-step workloads (paged KV caches, queries, block-size tables).

This module only *draws inputs*.  It contains none of the method's arithmetic (no
centroids, no quantization, no scoring, no selection, no attention, no derived sizes
such as centroid counts or per-head K): those live, separately and independently, in
the CPU oracle and in the HIP library.  Both sides are fed the arrays produced here.

The caches stand in for the Llama-3.1-8B / Qwen3 KV caches the paper measures on
(Sec. 4.1 "Hardware and models"): only the shapes are taken from there (query/KV head
counts, head_dim 128, context lengths 4K-128K, token budgets of a few percent, block
sizes 8..128 with mean near 32); every value is synthetic.

K/V/q are stored as uint16 bit patterns (IEEE binary16 or bfloat16) so the same bytes
can be handed to a C program and to the GPU without any dtype support on the way.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, Optional, Sequence

import numpy as np

F16 = 0
BF16 = 1


# --------------------------------------------------------------------------- formats
def f32_to_bits(x: np.ndarray, dtype: int) -> np.ndarray:
    """Round fp32 values to the storage format (round-to-nearest-even), return uint16 bits."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == F16:
        return x.astype(np.float16).view(np.uint16)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bits_to_f32(bits: np.ndarray, dtype: int) -> np.ndarray:
    """Exact widening of the stored uint16 bit patterns to fp32."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    if dtype == F16:
        return bits.view(np.float16).astype(np.float32)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------- container
@dataclass
class Workload:
    name: str
    dtype: int                      # F16 or BF16 (q, K, V share it)
    batch: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    page_size: int
    seq_lens: np.ndarray            # int32 [batch]
    budget: np.ndarray              # int32 [batch], token budget per KV head
    block_size: np.ndarray          # int32 [num_kv_heads]
    page_table: np.ndarray          # int32 [batch, pt_stride], logical -> physical page
    num_pages: int
    q: np.ndarray                   # uint16 [batch, Hq, d]
    k_cache: np.ndarray             # uint16 [num_pages, Hkv, P, d]  ("HND" pages)
    v_cache: np.ndarray             # uint16 [num_pages, Hkv, P, d]
    planted: Dict = field(default_factory=dict)   # (b, h) -> int64 array of heavy token positions
    knobs: Dict = field(default_factory=dict)     # the recipe's free parameters, for the report

    @property
    def group(self) -> int:
        return self.num_q_heads // self.num_kv_heads

    @property
    def strides(self):
        """(page, head, token) strides of the caches in elements."""
        P, d, H = self.page_size, self.head_dim, self.num_kv_heads
        return (H * P * d, P * d, d)

    def kv_bytes(self) -> int:
        return int(self.k_cache.nbytes + self.v_cache.nbytes)

    def key_rows(self, b: int, h: int) -> np.ndarray:
        """Logical [L_b, d] fp32 key matrix of (request b, KV head h): gathers through the page table."""
        return self._rows(self.k_cache, b, h)

    def value_rows(self, b: int, h: int) -> np.ndarray:
        return self._rows(self.v_cache, b, h)

    def _rows(self, cache, b, h):
        L = int(self.seq_lens[b])
        P = self.page_size
        npg = (L + P - 1) // P
        phys = self.page_table[b, :npg]
        rows = cache[phys, h].reshape(npg * P, self.head_dim)[:L]
        return bits_to_f32(rows, self.dtype)


def _streams(seed: int, n: int = 5):
    """Child streams in fixed order: block sizes, page permutation, lengths, data, planting."""
    return [np.random.Generator(np.random.PCG64(s)) for s in np.random.SeedSequence(seed).spawn(n)]


def _page_table(rng, seq_lens, P, shuffle: bool):
    npages = [(int(L) + P - 1) // P for L in seq_lens]
    total = int(sum(npages))
    perm = rng.permutation(total).astype(np.int32) if shuffle else np.arange(total, dtype=np.int32)
    pt = np.zeros((len(seq_lens), max(npages)), dtype=np.int32)
    o = 0
    for b, n in enumerate(npages):
        pt[b, :n] = perm[o:o + n]
        o += n
    return pt, total


def _scatter_rows(cache, pt_row, h, P, positions, rows_bits):
    """Overwrite logical tokens `positions` of head h with the given rows (uint16 bits)."""
    positions = np.asarray(positions, dtype=np.int64)
    cache[pt_row[positions // P], h, positions % P] = rows_bits


def _parallel_chunks(rng, n_items, chunk, work):
    """Run work(child_generator, lo, hi) over [0, n_items) in chunks on a thread pool.  Each chunk
    draws from its own spawned child stream, so the result does not depend on the thread count."""
    starts = list(range(0, n_items, chunk))
    kids = rng.bit_generator.seed_seq.spawn(len(starts))

    def run(i):
        g = np.random.Generator(np.random.PCG64(kids[i]))
        work(g, starts[i], min(n_items, starts[i] + chunk))

    with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
        list(ex.map(run, range(len(starts))))


def _fill_normal(rng, cache, dtype, scale=1.0, chunk_pages=128):
    """cache[...] <- N(0, scale^2) rounded to the storage format, generated in bounded chunks."""
    def work(g, p0, p1):
        x = g.standard_normal(size=(p1 - p0,) + cache.shape[1:], dtype=np.float32)
        if scale != 1.0:
            x *= np.float32(scale)
        cache[p0:p1] = f32_to_bits(x, dtype)

    _parallel_chunks(rng, cache.shape[0], chunk_pages, work)


def _unit_rms_direction(rng, d, unit):
    g = rng.standard_normal(d)
    g /= np.linalg.norm(g)
    if unit == "rms":            # ||u||_2 = sqrt(d): every component has unit RMS
        g *= np.sqrt(d)
    return g.astype(np.float32)  # unit == "l2": ||u||_2 = 1


def _plant_fixed(rng, wl: Workload, q32, n_plant, gain, unit):
    """Config-1 style planting: per (request, KV head) `n_plant` keys are replaced by
    gain*u (u a random direction), and u is added to every query head of the group."""
    G, P = wl.group, wl.page_size
    for b in range(wl.batch):
        L = int(wl.seq_lens[b])
        for h in range(wl.num_kv_heads):
            u = _unit_rms_direction(rng, wl.head_dim, unit)
            pos = np.sort(rng.choice(L, size=min(n_plant, L), replace=False))
            rows = np.broadcast_to(f32_to_bits(gain * u, wl.dtype), (len(pos), wl.head_dim))
            _scatter_rows(wl.k_cache, wl.page_table[b], h, P, pos, rows)
            q32[b, h * G:(h + 1) * G] += u
            wl.planted[(b, h)] = pos.astype(np.int64)


def _plant_zipf(rng, wl: Workload, q32, n_heavy, z_top, exponent, run_choices, run_lengths=None):
    """Config-3 style planting.  Per (request, KV head): `n_heavy` heavy tokens ranked
    r = 1..n_heavy get a target logit z_r = z_top - exponent*ln r along the group-mean
    query direction, so their dense-softmax mass falls off as r^-exponent.  Heavy tokens
    sit in runs of rho consecutive positions (rho drawn per head: clustered vs scattered
    heads, Sec. 2.3 of the paper)."""
    G, P, d = wl.group, wl.page_size, wl.head_dim
    sm = 1.0 / np.sqrt(d)
    rho_of_head = rng.choice(np.asarray(run_choices), size=wl.num_kv_heads)
    if run_lengths is not None:       # fixed head roles (the draw above is still taken: the streams stay aligned)
        rho_of_head = np.asarray(run_lengths, dtype=rho_of_head.dtype)
        assert rho_of_head.shape == (wl.num_kv_heads,)
    wl.knobs["run_length"] = [int(x) for x in rho_of_head]
    for b in range(wl.batch):
        L = int(wl.seq_lens[b])
        for h in range(wl.num_kv_heads):
            rho = int(rho_of_head[h])
            M = min(n_heavy, (L // 2 // rho) * rho)
            if M <= 0:
                continue
            nruns = M // rho
            # run starts: distinct rho-aligned slots, uniform over the context
            slots = rng.choice(L // rho, size=nruns, replace=False)
            pos = (slots[:, None] * rho + np.arange(rho)[None, :]).reshape(-1)
            pos = pos[rng.permutation(pos.size)]            # rank r -> position pos[r-1]
            qbar = q32[b, h * G:(h + 1) * G].mean(axis=0)
            nq = float(np.linalg.norm(qbar))
            uhat = (qbar / nq).astype(np.float32)
            z = z_top - exponent * np.log(np.arange(1, M + 1))
            beta = (z / (sm * nq)).astype(np.float32)
            noise = rng.standard_normal(size=(M, d), dtype=np.float32)
            rows = noise + beta[:, None] * uhat[None, :]
            _scatter_rows(wl.k_cache, wl.page_table[b], h, P, pos, f32_to_bits(rows, wl.dtype))
            wl.planted[(b, h)] = np.sort(pos).astype(np.int64)


def _empty(name, dtype, Bt, Hq, Hkv, d, P, seq_lens, budget, block_size, page_table, num_pages):
    return Workload(
        name=name, dtype=dtype, batch=Bt, num_q_heads=Hq, num_kv_heads=Hkv, head_dim=d, page_size=P,
        seq_lens=np.asarray(seq_lens, dtype=np.int32), budget=np.asarray(budget, dtype=np.int32),
        block_size=np.asarray(block_size, dtype=np.int32), page_table=page_table, num_pages=num_pages,
        q=np.zeros((Bt, Hq, d), dtype=np.uint16),
        k_cache=np.zeros((num_pages, Hkv, P, d), dtype=np.uint16),
        v_cache=np.zeros((num_pages, Hkv, P, d), dtype=np.uint16))


# --------------------------------------------------------------------------- recipes
def make_workload(config: int, *, seed: Optional[int] = None, context: Optional[int] = None,
                  batch: Optional[int] = None, budget: Optional[int] = None,
                  block_sizes: Optional[Sequence[int]] = None, uniform_block: Optional[int] = None,
                  shuffle_pages: bool = True, plant_unit: str = "rms",
                  seq_lens: Optional[Sequence[int]] = None,
                  run_lengths: Optional[Sequence[int]] = None,
                  head_block_sizes: Optional[Sequence[int]] = None) -> Workload:
    """Build one of the five benchmark-shaped workloads (1-based `config`), optionally
    scaled down (context / batch / budget overrides) for quick tests.

    1: B1, 32/8 heads, L=4096, fp16, block sizes from {8,16,32,64}, T=512, 16 planted keys/head, seed 0
    2: B8, 32/8, L=32768, bf16, low-rank keys (rank 8 + 0.1 noise), {16,32,64}, T=2048, seed 1
    3: B1, 32/8, L=131072, fp16, Zipf(1.1) heavy tokens, {8,...,128}, T=4096, seed 2   (headline)
    4: B16, 40/8, L~U[8192,131072], bf16, {16,32,64}, T=ceil(3% L), planted as 1, seed 3
    5: B4, 32/8, L=65536, fp16, uniform 16 or adaptive {8,...,128}, T swept by the caller, seed 4
    """
    d, P, Hkv = 128, 64, 8
    defaults = {
        1: dict(seed=0, Bt=1, Hq=32, L=4096, dtype=F16, sizes=(8, 16, 32, 64), T=512),
        2: dict(seed=1, Bt=8, Hq=32, L=32768, dtype=BF16, sizes=(16, 32, 64), T=2048),
        3: dict(seed=2, Bt=1, Hq=32, L=131072, dtype=F16, sizes=(8, 16, 32, 64, 128), T=4096),
        4: dict(seed=3, Bt=16, Hq=40, L=None, dtype=BF16, sizes=(16, 32, 64), T=None),
        5: dict(seed=4, Bt=4, Hq=32, L=65536, dtype=F16, sizes=(8, 16, 32, 64, 128), T=4096),
    }[config]
    seed = defaults["seed"] if seed is None else seed
    Bt = defaults["Bt"] if batch is None else batch
    Hq, dtype = defaults["Hq"], defaults["dtype"]
    sizes = tuple(block_sizes) if block_sizes is not None else defaults["sizes"]
    r_bs, r_pg, r_len, r_data, r_plant = _streams(seed)

    bs = r_bs.choice(np.asarray(sizes), size=Hkv).astype(np.int32)
    if uniform_block is not None:
        bs[:] = uniform_block
    if head_block_sizes is not None:           # an explicit assignment (a calibration's result), one size per KV head
        bs = np.asarray(head_block_sizes, dtype=np.int32).reshape(Hkv).copy()

    if seq_lens is not None:
        lens = np.asarray(seq_lens, dtype=np.int32)
        Bt = len(lens)
    elif config == 4:
        hi = 131072 if context is None else context
        lo = max(1, hi // 16)
        lens = r_len.integers(lo, hi + 1, size=Bt).astype(np.int32)
    else:
        lens = np.full(Bt, defaults["L"] if context is None else context, dtype=np.int32)

    if budget is not None:
        T = np.full(Bt, budget, dtype=np.int32)
    elif config == 4:
        T = ((3 * lens.astype(np.int64) + 99) // 100).astype(np.int32)     # ceil(0.03 L)
    else:
        T = np.full(Bt, defaults["T"], dtype=np.int32)

    pt, total_pages = _page_table(r_pg, lens, P, shuffle_pages)
    wl = _empty(f"config{config}", dtype, Bt, Hq, Hkv, d, P, lens, T, bs, pt, total_pages)
    wl.knobs.update(seed=seed, shuffle_pages=shuffle_pages, block_size_set=list(sizes))

    q32 = r_data.standard_normal(size=(Bt, Hq, d), dtype=np.float32)
    _fill_normal(r_data, wl.v_cache, dtype)
    if config == 2:
        # keys = coefficients x per-head rank-8 basis + 0.1 * noise
        W = (r_data.standard_normal(size=(Hkv, 8, d)) / np.sqrt(8.0)).astype(np.float32)

        def work(g, p0, p1):
            C = g.standard_normal(size=(p1 - p0, Hkv, P, 8), dtype=np.float32)
            x = np.einsum("phtr,hrd->phtd", C, W, optimize=True)
            x += np.float32(0.1) * g.standard_normal(size=x.shape, dtype=np.float32)
            wl.k_cache[p0:p1] = f32_to_bits(x.astype(np.float32), dtype)

        _parallel_chunks(r_data, total_pages, 128, work)
        wl.knobs.update(key_rank=8, key_noise=0.1)
    else:
        _fill_normal(r_data, wl.k_cache, dtype)

    if config in (1, 4):
        _plant_fixed(r_plant, wl, q32, n_plant=16, gain=4.0, unit=plant_unit)
        wl.knobs.update(planting="fixed", n_plant=16, gain=4.0, unit=plant_unit)
    elif config in (3, 5):
        _plant_zipf(r_plant, wl, q32, n_heavy=4096, z_top=16.0, exponent=1.1, run_choices=(1, 4, 16, 64),
                    run_lengths=run_lengths)
        wl.knobs.update(planting="zipf", n_heavy=4096, z_top=16.0, exponent=1.1)
    wl.q = f32_to_bits(q32, dtype)
    return wl


def tiny_workload(*, seed=0, dtype=F16, Bt=2, Hq=8, Hkv=2, d=128, P=16, seq_lens=(37, 64),
                  block_size=(8, 32), budget=(16, 24), shuffle_pages=True, extra_pages=3) -> Workload:
    """A small free-form workload for unit tests: ragged lengths, any page size, spare
    (unused) physical pages so that a wrong page lookup lands on different data."""
    r_pg, r_data = [np.random.Generator(np.random.PCG64(s)) for s in np.random.SeedSequence(seed).spawn(2)]
    lens = np.asarray(seq_lens, dtype=np.int32)
    Bt = len(lens)
    npages = [(int(L) + P - 1) // P for L in lens]
    total = int(sum(npages)) + extra_pages
    perm = r_pg.permutation(total).astype(np.int32) if shuffle_pages else np.arange(total, dtype=np.int32)
    pt = np.zeros((Bt, max(npages) + 1), dtype=np.int32)
    o = 0
    for b, n in enumerate(npages):
        pt[b, :n] = perm[o:o + n]
        o += n
    wl = _empty("tiny", dtype, Bt, Hq, Hkv, d, P, lens, np.broadcast_to(np.asarray(budget, np.int32), (Bt,)).copy(),
                np.broadcast_to(np.asarray(block_size, np.int32), (Hkv,)).copy(), pt, total)
    _fill_normal(r_data, wl.k_cache, dtype)
    _fill_normal(r_data, wl.v_cache, dtype)
    wl.q = f32_to_bits(r_data.standard_normal(size=(Bt, Hq, d), dtype=np.float32), dtype)
    wl.knobs.update(seed=seed)
    return wl
