"""Seeded synthetic step batches for the mixed prefill/decode paged-attention path.

This module only *makes inputs*: request lengths, block tables, bf16 bit
patterns for Q and for the KV page pool.  It holds none of the attention
arithmetic and is the one module both the HIP path's tests/bench and the CPU
oracle's tests draw inputs from.  It depends on numpy only.

The five named configurations follow the serving-shaped batches the library is
measured on (one scheduled step as Section 3.3.1 of the HFX paper states it:
in-flight decodes plus admitted prompt chunks, heterogeneous lengths as in
Table 1).  No dataset item is reproduced: attention cost depends on lengths
only, so lengths are drawn from distributions and all values are N(0,1).

Pool layout written here (bf16 bits, uint16): pool[page][kv_head][0] holds the
keys blocked by 16 dimensions, viewed as [D/16][16 slots][16] (element (slot, d)
at ((d//16)*16 + slot)*16 + d%16); pool[page][kv_head][1] holds the values
dimension-major, viewed as [D][16 slots].
"""
from __future__ import annotations

import math
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field

import numpy as np

PAGE = 16
DECODE = 0
PREFILL = 1
BF16_NAN = np.uint16(0x7FC0)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns.

    Inputs are finite here, so no NaN quieting is needed.
    """
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) exactly to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) exactly to float64."""
    return bf16_bits_to_f32(b).astype(np.float64)


@dataclass
class StepBatch:
    """One scheduled step: per-request records, block table, Q and the page pool."""

    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    num_pages: int
    kind: np.ndarray        # int32 [R]
    q_len: np.ndarray       # int32 [R]
    ctx_len: np.ndarray     # int32 [R]
    bt_indptr: np.ndarray   # int32 [R+1]
    bt_pages: np.ndarray    # int32 [bt_indptr[R]]
    q: np.ndarray           # uint16 [T, Hq, D]
    pool: np.ndarray        # uint16 [num_pages, Hkv, 2, 16*D]
    name: str = ""
    notes: dict = field(default_factory=dict)

    @property
    def num_requests(self) -> int:
        return int(self.kind.shape[0])

    @property
    def total_q(self) -> int:
        return int(self.q_len.sum())

    def pool_shape(self):
        return (self.num_pages, self.num_kv_heads, 2, PAGE * self.head_dim)

    def q_indptr(self) -> np.ndarray:
        out = np.zeros(self.num_requests + 1, dtype=np.int64)
        np.cumsum(self.q_len, out=out[1:])
        return out

    # ---- algorithmic work of the step (what the method itself must move / compute)
    def decode_kv_bytes(self) -> int:
        dec = self.kind == DECODE
        toks = int(self.ctx_len[dec].astype(np.int64).sum())
        return toks * self.num_kv_heads * self.head_dim * 2 * 2

    def decode_io_bytes(self) -> int:
        """KV bytes plus Q in and out for the decode requests."""
        ndec = int((self.kind == DECODE).sum())
        return self.decode_kv_bytes() + ndec * 2 * self.num_q_heads * self.head_dim * 2

    def prefill_pairs(self) -> int:
        pre = self.kind == PREFILL
        q = self.q_len[pre].astype(np.int64)
        p = self.ctx_len[pre].astype(np.int64) - q
        return int((q * p + q * (q + 1) // 2).sum())

    def prefill_flops(self) -> int:
        return 4 * self.head_dim * self.num_q_heads * self.prefill_pairs()

    def prefill_io_bytes(self) -> int:
        pre = self.kind == PREFILL
        c = int(self.ctx_len[pre].astype(np.int64).sum())
        q = int(self.q_len[pre].astype(np.int64).sum())
        return c * self.num_kv_heads * self.head_dim * 2 * 2 + q * 2 * self.num_q_heads * self.head_dim * 2

    def sub_batch(self, which: int) -> "StepBatch":
        """The decode-only (which=DECODE) or prefill-only (which=PREFILL) part of the step,
        over the same pool and pages."""
        sel = np.nonzero(self.kind == which)[0]
        qi = self.q_indptr()
        rows = np.concatenate([np.arange(qi[r], qi[r + 1]) for r in sel]) if len(sel) else np.zeros(0, np.int64)
        segs = [self.bt_pages[self.bt_indptr[r]:self.bt_indptr[r + 1]] for r in sel]
        indptr = np.zeros(len(sel) + 1, dtype=np.int32)
        if len(sel):
            indptr[1:] = np.cumsum([len(s) for s in segs])
        return StepBatch(
            self.num_q_heads, self.num_kv_heads, self.head_dim, self.num_pages,
            self.kind[sel].copy(), self.q_len[sel].copy(), self.ctx_len[sel].copy(), indptr,
            np.concatenate(segs).astype(np.int32) if len(sel) else np.zeros(0, np.int32),
            np.ascontiguousarray(self.q[rows]), self.pool,
            name=self.name + ("/decode" if which == DECODE else "/prefill"), notes=dict(self.notes))


def _n_threads() -> int:
    try:
        n = int(os.environ.get("OMP_NUM_THREADS", "0"))
    except ValueError:
        n = 0
    if n <= 0:
        n = min(os.cpu_count() or 1, 16)
    return max(1, min(n, 16))


def _normal_bf16(seed_words, n: int) -> np.ndarray:
    g = np.random.Generator(np.random.PCG64(np.random.SeedSequence(list(seed_words))))
    return f32_to_bf16_bits(g.standard_normal(n, dtype=np.float32))


def _fill_pool_normal(pool: np.ndarray, pages: np.ndarray, seed: int) -> None:
    """Fill the listed physical pages with N(0,1) bf16 bits, in parallel, deterministically.

    The value of a page depends on (seed, position of the page in `pages`), not on
    the physical id, so re-shuffling the pool moves data without changing it.
    """
    per_page = pool[0].size
    chunk = max(1, (8 << 20) // per_page)
    jobs = [(i, min(i + chunk, len(pages))) for i in range(0, len(pages), chunk)]

    def run(job):
        a, b = job
        vals = _normal_bf16((seed, 0x706F6F6C, a), (b - a) * per_page)
        pool.reshape(pool.shape[0], per_page)[pages[a:b]] = vals.reshape(b - a, per_page)

    if len(jobs) <= 1:
        for j in jobs:
            run(j)
    else:
        with ThreadPoolExecutor(_n_threads()) as ex:
            list(ex.map(run, jobs))


def poison_tails(batch: StepBatch) -> None:
    """Overwrite the unused slots [ctx_len % 16, 16) of every request's last page with NaN.

    A page shared by two requests is only poisoned past the longest context that reads it.
    """
    d = batch.head_dim
    reach = {}
    for r in range(batch.num_requests):
        c = int(batch.ctx_len[r])
        npg = (c + PAGE - 1) // PAGE
        seg = batch.bt_pages[batch.bt_indptr[r]:batch.bt_indptr[r] + npg]
        for i, p in enumerate(seg):
            used = min(PAGE, c - i * PAGE)
            reach[int(p)] = max(reach.get(int(p), 0), used)
    for p, used in reach.items():
        if used < PAGE:
            k = batch.pool[p, :, 0].reshape(batch.num_kv_heads, d // 16, PAGE, 16)
            v = batch.pool[p, :, 1].reshape(batch.num_kv_heads, d, PAGE)
            k[:, :, used:, :] = BF16_NAN
            v[:, :, used:] = BF16_NAN


def make_batch(num_q_heads: int, num_kv_heads: int, head_dim: int, kind, q_len, ctx_len,
               seed: int, over_provision: float = 1.25, extra_pages_per_request: int = 0,
               name: str = "", poison: bool = True, fill_pool: bool = True) -> StepBatch:
    """Build a step over a shuffled, over-provisioned page pool.

    Physical ids are the first `need` entries of a seeded permutation of
    [0, num_pages), num_pages = ceil(over_provision * need).  Unused pages and
    last-page tails are NaN when `poison`.  `extra_pages_per_request` appends
    reserved-but-unused (poisoned) pages to each block table.  With `fill_pool=False`
    only lengths, block table and Q are made and `pool` is None (the caller fills a
    device-resident pool of shape pool_shape() itself).
    """
    kind = np.asarray(kind, dtype=np.int32)
    q_len = np.asarray(q_len, dtype=np.int32)
    ctx_len = np.asarray(ctx_len, dtype=np.int32)
    R = len(kind)
    g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 0x73746570])))
    npg = (ctx_len.astype(np.int64) + PAGE - 1) // PAGE
    per_req = npg + extra_pages_per_request
    need = int(per_req.sum())
    num_pages = max(1, int(math.ceil(over_provision * need)))
    perm = g.permutation(num_pages).astype(np.int32)
    bt_pages = perm[:need].copy()
    bt_indptr = np.zeros(R + 1, dtype=np.int32)
    bt_indptr[1:] = np.cumsum(per_req)
    pool = None
    if fill_pool:
        pool = np.empty((num_pages, num_kv_heads, 2, PAGE * head_dim), dtype=np.uint16)
        pool[...] = BF16_NAN if poison else 0
        used = np.concatenate([bt_pages[bt_indptr[r]:bt_indptr[r] + npg[r]] for r in range(R)]) if R else bt_pages
        _fill_pool_normal(pool, used, seed)
    T = int(q_len.sum())
    q = _normal_bf16((seed, 0x71), T * num_q_heads * head_dim).reshape(T, num_q_heads, head_dim)
    b = StepBatch(num_q_heads, num_kv_heads, head_dim, num_pages, kind, q_len, ctx_len,
                  bt_indptr, bt_pages, q, pool, name=name)
    if poison and fill_pool:
        poison_tails(b)
    return b


def permute_pages(batch: StepBatch, seed: int) -> StepBatch:
    """The same logical step with every physical page moved: data follow their pages and
    the block table is rewritten."""
    g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 0x7065726D])))
    new_of_old = g.permutation(batch.num_pages).astype(np.int32)
    pool = np.empty_like(batch.pool)
    pool[new_of_old] = batch.pool
    return StepBatch(batch.num_q_heads, batch.num_kv_heads, batch.head_dim, batch.num_pages,
                     batch.kind.copy(), batch.q_len.copy(), batch.ctx_len.copy(), batch.bt_indptr.copy(),
                     new_of_old[batch.bt_pages], batch.q.copy(), pool, name=batch.name + "/permuted",
                     notes=dict(batch.notes))


# ---------------------------------------------------------------------------------------
# The five named configurations.  `scale` < 1 shrinks request counts and lengths for
# parity runs the CPU oracle finishes in seconds; scale == 1 is the full size.
# ---------------------------------------------------------------------------------------

def _scaled(n: int, scale: float, lo: int = 1) -> int:
    return max(lo, int(round(n * scale)))


def config(index: int, scale: float = 1.0, seed: int | None = None, fill_pool: bool = True) -> StepBatch:
    """Configuration `index` (1-based).  Seed defaults to index-1."""
    if seed is None:
        seed = index - 1
    g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 0x6C656E])))
    if index == 1:
        # 3 decodes (context 37/64/129) + 1 prompt chunk of 32 whose context is the chunk itself.
        b = make_batch(4, 2, 64, [DECODE, DECODE, DECODE, PREFILL], [1, 1, 1, 32], [37, 64, 129, 32],
                       seed, name="cfg1-tiny-mixed", fill_pool=fill_pool)
    elif index == 2:
        nd = _scaled(64, scale)
        cap = _scaled(8192, scale, 64)
        med = _scaled(1024, scale, 16)
        c = np.clip(np.rint(np.exp(g.normal(math.log(med), 1.0, nd))), 16, cap).astype(np.int32)
        ch = _scaled(512, scale, 16)
        kinds = [DECODE] * nd + [PREFILL, PREFILL]
        b = make_batch(32, 8, 128, kinds, list(np.ones(nd, np.int32)) + [ch, ch],
                       list(c) + [ch, 4 * ch], seed, name="cfg2-llama8b-mixed", fill_pool=fill_pool)
    elif index == 3:
        nd = _scaled(256, scale)
        lo, hi = _scaled(2048, scale, 16), _scaled(16384, scale, 64)
        c = g.integers(lo, hi + 1, nd).astype(np.int32)
        b = make_batch(32, 8, 128, [DECODE] * nd, np.ones(nd, np.int32), c, seed, name="cfg3-decode-heavy", fill_pool=fill_pool)
    elif index == 4:
        ch = _scaled(2048, scale, 32)
        nd = _scaled(32, scale, 2)
        base = _scaled(2048, scale, 64)
        jit = max(1, base // 8)
        cd = (base + g.integers(-jit, jit + 1, nd)).astype(np.int32)
        prior = [0, 2 * ch, 4 * ch, 6 * ch]
        kinds = [PREFILL] * 4 + [DECODE] * nd
        b = make_batch(32, 8, 128, kinds, [ch] * 4 + [1] * nd, [p + ch for p in prior] + list(cd),
                       seed, name="cfg4-prefill-heavy", fill_pool=fill_pool)
    elif index == 5:
        nd = _scaled(16, scale, 2)
        lo, hi = _scaled(32768, scale, 64), _scaled(131072, scale, 256)
        cd = g.integers(lo, hi + 1, nd).astype(np.int32)
        ch = _scaled(4096, scale, 32)
        ctx = _scaled(65536, scale, ch)
        kinds = [DECODE] * nd + [PREFILL]
        b = make_batch(8, 1, 128, kinds, [1] * nd + [ch], list(cd) + [max(ctx, ch)], seed,
                       name="cfg5-long-context-tp-share", fill_pool=fill_pool)
    else:
        raise ValueError("config index must be 1..5")
    b.notes.update(config=index, scale=scale, seed=seed)
    return b


def table1_short_context(seed: int = 7, requests_per_task: int = 16) -> StepBatch:
    """A short-context step shaped like Table 1 of the paper: per task, prompt lengths
    ~N(mean, std) clipped to >= 4, half of the requests still prefilling their whole prompt
    and half decoding at prompt + U[1, mean output] tokens."""
    g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 0x7431])))
    tasks = [(32.6, 10.3, 38.9), (44.4, 6.6, 96.0), (121.8, 35.0, 13.6),
             (643.2, 337.0, 27.8), (51.4, 15.8, 90.1), (259.2, 324.9, 207.8)]
    kinds, ql, cl = [], [], []
    for mean, std, out in tasks:
        lens = np.maximum(4, np.rint(g.normal(mean, std, requests_per_task))).astype(np.int64)
        for i, n in enumerate(lens):
            if i % 2 == 0:
                kinds.append(PREFILL); ql.append(int(n)); cl.append(int(n))
            else:
                kinds.append(DECODE); ql.append(1); cl.append(int(n + g.integers(1, max(2, int(out)) + 1)))
    return make_batch(32, 8, 128, kinds, ql, cl, seed, name="table1-short-context")
