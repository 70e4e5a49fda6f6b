"""Seeded synthetic decode batches shaped like the paper's DCP workloads.

A batch is what ONE KV-binding instance sees in one decode step (paper: Data Plane,
Phase 2 inputs in Alg. 2 -- routed queries, block table, attention lengths, local paged KV)
plus the bookkeeping Phase 4 needs to merge a long request's partials.  The generators
only draw random numbers and lay them out in memory; they contain no attention arithmetic.
Both the float64 checker and the GPU library consume the very same raw buffers.

Storage layouts (x = 16 bytes / sizeof(kv element): 4 for f32, 8 for bf16, 16 for fp8):
  q            [q_rows, Hq, Dk]                       f32, or bf16 bit patterns (uint16)
  GQA k_pool   [pages, Hkv, ps/4x, Dk/x, 4x, x]       token groups of 4x slots; inside a group, 16-byte vectors of
                                                      x dims, token-major inside a dim chunk
  GQA v_pool   [pages, Hkv, ps/x, Dv, x]              16-byte vectors of x tokens of one dim.  Inside every group of
                                                      4x tokens, slot w = 16b + 4g + i (i < 4, g < 4) is element 4b + i
                                                      of the group's vector g  (for f32, x = 4, that is plain order)
  MLA k_pool   [pages, ps, Dk]                        one latent row per token; V is its first Dv dims
  k_scale/v_scale [pages, Hkv] f32                    fp8 only
  block_table  [rows, max_blocks] int32               physical page ids, -1 past a row's last page
  shards       [S, 4] int32                           (q_row, bt_row, kv_begin, kv_end), tokens relative to the row's page 0
Slots of allocated pages that hold no token of the row, and spare pages, are filled with NaN
patterns so that a kernel that fails to mask them is caught.
"""
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

from . import numfmt

KV_ELEM_BYTES = {"f32": 4, "bf16": 2, "fp8": 1}


@dataclass
class AttnDesc:
    kind: str            # "gqa" | "mla"
    q_dtype: str         # "f32" | "bf16"
    kv_dtype: str        # "f32" | "bf16" | "fp8"
    num_q_heads: int
    num_kv_heads: int
    head_dim_qk: int
    head_dim_v: int
    page_size: int
    softmax_scale: float

    @property
    def vec(self):
        return 16 // KV_ELEM_BYTES[self.kv_dtype]

    @property
    def kv_bytes_per_token(self):
        e = KV_ELEM_BYTES[self.kv_dtype]
        if self.kind == "mla":
            return self.head_dim_qk * e
        return self.num_kv_heads * (self.head_dim_qk + self.head_dim_v) * e


@dataclass
class RemoteShard:
    """KV of a shard that another instance would hold (host only, for the checker)."""
    request: int
    q_row: int
    k_pool: np.ndarray
    v_pool: Optional[np.ndarray]
    k_scale: Optional[np.ndarray]
    v_scale: Optional[np.ndarray]
    block_table: np.ndarray       # [1, blocks]
    kv_begin: int
    kv_end: int


@dataclass
class Batch:
    name: str
    seed: int
    desc: AttnDesc
    q: np.ndarray
    k_pool: np.ndarray
    v_pool: Optional[np.ndarray]
    k_scale: Optional[np.ndarray]
    v_scale: Optional[np.ndarray]
    block_table: np.ndarray
    shards: np.ndarray                       # [S,4] int32
    lengths: np.ndarray                      # [R] full request lengths
    cp_degree: np.ndarray                    # [R]
    ranges: List[List[tuple]]                # per request: its d token ranges in request coordinates
    part_offsets: np.ndarray                 # [R+1] int32
    part_index: np.ndarray                   # [Ptot] int32; < S: local shard entry, >= S: remotes[idx-S]
    remote_meta: List[tuple]                 # (request, q_row, begin, end) per remote shard, always present
    remotes: List[RemoteShard] = field(default_factory=list)   # filled only if with_remote_kv

    @property
    def num_shards(self):
        return int(self.shards.shape[0])

    @property
    def num_requests(self):
        return int(self.lengths.shape[0])

    @property
    def local_tokens(self):
        return int((self.shards[:, 3] - self.shards[:, 2]).sum())

    @property
    def kv_bytes(self):
        """Algorithmic KV bytes one decode step must read on this GPU (scales included for fp8)."""
        d = self.desc
        b = self.local_tokens * d.kv_bytes_per_token
        if d.kv_dtype == "fp8":
            pages = 0
            for _, _, b0, e0 in self.shards:
                if e0 > b0:
                    pages += (int(e0) - 1) // d.page_size - int(b0) // d.page_size + 1
            b += pages * d.num_kv_heads * 8
        return int(b)


# --------------------------------------------------------------------------- pool drawing

def _pool_shapes(desc, pages):
    x, ps = desc.vec, desc.page_size
    if desc.kind == "mla":
        return (pages, ps, desc.head_dim_qk), None
    assert desc.head_dim_qk % x == 0 and ps % (4 * x) == 0
    return ((pages, desc.num_kv_heads, ps // (4 * x), desc.head_dim_qk // x, 4 * x, x),
            (pages, desc.num_kv_heads, ps // x, desc.head_dim_v, x))


def v_slot(slot, x):
    """(vector index, element) of a token slot inside a page of the V layout."""
    grp, w = divmod(slot, 4 * x)
    return grp * 4 + (w % 16) // 4, 4 * (w // 16) + w % 4


def _draw_f32(rng, shape):
    return rng.standard_normal(size=shape, dtype=np.float32)


def _poison_slots(desc, k, v, page, lo, hi):
    """Mark token slots [lo,hi) of physical page `page` as unused (NaN patterns)."""
    if hi <= lo:
        return
    if desc.kv_dtype == "f32":
        nan = np.float32(np.nan)
    elif desc.kv_dtype == "bf16":
        nan = numfmt.BF16_NAN
    else:
        nan = numfmt.FP8_NAN
    x = desc.vec
    if desc.kind == "mla":
        k[page, lo:hi, :] = nan
        return
    for t in range(lo, hi):
        k[page, :, t // (4 * x), :, t % (4 * x), :] = nan
        u, e = v_slot(t, x)
        v[page, :, u, :, e] = nan


def _encode_pool(desc, raw):
    """float32 draws -> stored element type (+ per-page-per-head scale for fp8)."""
    if desc.kv_dtype == "f32":
        return raw, None
    if desc.kv_dtype == "bf16":
        return numfmt.f32_to_bf16_bits(raw), None
    return numfmt.quantize_per_page_head(raw, desc.num_kv_heads)


POOL_CHUNK_PAGES = 128


def _draw_pool(desc, seed, tag, pages):
    """Draw K (and V) pools of `pages` pages.  The pool is drawn in chunks of POOL_CHUNK_PAGES
    pages; chunk c of pool `tag` uses default_rng([seed, tag, which, c]) (which: 0=K, 1=V), so the
    content does not depend on how many worker threads fill it."""
    ks, vs = _pool_shapes(desc, pages)
    store = {"f32": np.float32, "bf16": np.uint16, "fp8": np.uint8}[desc.kv_dtype]
    out = []
    jobs = []
    for which, shape in ((0, ks), (1, vs)):
        if shape is None:
            out.append((None, None))
            continue
        pool = np.empty(shape, store)
        scale = np.empty((pages, desc.num_kv_heads), np.float32) if desc.kv_dtype == "fp8" else None
        out.append((pool, scale))
        for c, p0 in enumerate(range(0, pages, POOL_CHUNK_PAGES)):
            jobs.append((which, c, p0, min(pages, p0 + POOL_CHUNK_PAGES), pool, scale))

    def fill(job):
        which, c, p0, p1, pool, scale = job
        rng = np.random.default_rng([seed, tag, which, c])
        enc, sc = _encode_pool(desc, _draw_f32(rng, (p1 - p0,) + pool.shape[1:]))
        pool[p0:p1] = enc
        if sc is not None:
            scale[p0:p1] = sc

    if len(jobs) <= 2:
        for j in jobs:
            fill(j)
    else:
        from concurrent.futures import ThreadPoolExecutor
        import os
        with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
            list(ex.map(fill, jobs))
    (k, k_scale), (v, v_scale) = out
    return k, v, k_scale, v_scale


def _encode_q(desc, qf):
    return qf if desc.q_dtype == "f32" else numfmt.f32_to_bf16_bits(qf)


# --------------------------------------------------------------------------- batch assembly

def build_batch(name, seed, desc, lengths, ranges, local, rng, with_remote_kv=True, spare_pages=3):
    """Assemble one instance's batch.

    lengths[r]        full KV length of request r
    ranges[r]         list of d_r token ranges [(b,e),...] covering [0,len) (the request's CP split)
    local[r]          indices into ranges[r] of the shards this GPU holds (possibly all of them)
    `rng` (already used for the lengths) then draws the block-table permutation and q; pool contents
    come from child generators keyed by (seed, pool tag, K/V, chunk) -- see _draw_pool.
    """
    ps = desc.page_size
    R = len(lengths)
    rows = []          # per block-table row: (request, first_token_offset, n_tokens)
    shard_list = []
    part_lists = [[] for _ in range(R)]
    remote_meta = []
    for r in range(R):
        d = len(ranges[r])
        all_local = len(local[r]) == d
        if all_local:
            row = len(rows)
            rows.append((r, 0, int(lengths[r])))
        for i, (b, e) in enumerate(ranges[r]):
            if i in local[r]:
                if all_local:
                    sh = (r, row, int(b), int(e))
                else:
                    off = int(b) % ps            # token-level split keeps the in-page offset of the cut
                    sh = (r, len(rows), off, off + int(e - b))
                    rows.append((r, off, int(e - b)))
                part_lists[r].append(len(shard_list))
                shard_list.append(sh)
            else:
                part_lists[r].append(-1 - len(remote_meta))
                remote_meta.append((r, r, int(b), int(e)))
    S = len(shard_list)
    part_offsets = np.zeros(R + 1, np.int32)
    part_index = []
    for r in range(R):
        for p in part_lists[r]:
            part_index.append(p if p >= 0 else S + (-1 - p))
        part_offsets[r + 1] = len(part_index)
    part_index = np.asarray(part_index, np.int32)

    row_pages = [(off + n + ps - 1) // ps if n > 0 else 0 for (_, off, n) in rows]
    row_pages = [max(p, 1) for p in row_pages]          # every row owns at least one page
    total_pages = int(sum(row_pages)) + spare_pages
    max_blocks = max(row_pages)
    perm = rng.permutation(total_pages).astype(np.int32)
    block_table = np.full((len(rows), max_blocks), -1, np.int32)
    cur = 0
    for i, n in enumerate(row_pages):
        block_table[i, :n] = perm[cur:cur + n]
        cur += n
    spare = perm[cur:]

    q = _encode_q(desc, _draw_f32(rng, (R, desc.num_q_heads, desc.head_dim_qk)))
    k_pool, v_pool, k_scale, v_scale = _draw_pool(desc, seed, 0, total_pages)
    for i, (_, off, n) in enumerate(rows):
        first, last = block_table[i, 0], block_table[i, row_pages[i] - 1]
        if row_pages[i] == 1:
            _poison_slots(desc, k_pool, v_pool, first, 0, off)
            _poison_slots(desc, k_pool, v_pool, first, off + n, ps)
        else:
            _poison_slots(desc, k_pool, v_pool, first, 0, off)
            _poison_slots(desc, k_pool, v_pool, last, (off + n - 1) % ps + 1, ps)
    for p in spare:
        _poison_slots(desc, k_pool, v_pool, p, 0, ps)

    remotes = []
    if with_remote_kv:
        for ri, (r, q_row, b, e) in enumerate(remote_meta):
            off = b % ps
            n = e - b
            pages = max((off + n + ps - 1) // ps, 1)
            rk, rv, rks, rvs = _draw_pool(desc, seed, 1 + ri, pages)
            _poison_slots(desc, rk, rv, 0, 0, off)
            if n > 0:
                _poison_slots(desc, rk, rv, pages - 1, (off + n - 1) % ps + 1, ps)
            remotes.append(RemoteShard(r, q_row, rk, rv, rks, rvs,
                                       np.arange(pages, dtype=np.int32)[None, :], off, off + n))

    return Batch(name, seed, desc, q, k_pool, v_pool, k_scale, v_scale, block_table,
                 np.asarray(shard_list, np.int32).reshape(S, 4), np.asarray(lengths, np.int64),
                 np.asarray([len(x) for x in ranges], np.int32), ranges, part_offsets, part_index,
                 remote_meta, remotes)


def even_split(length, d):
    """CP split used by the generators: b_i = floor(i*L/d)."""
    cuts = [(i * int(length)) // d for i in range(d + 1)]
    return [(cuts[i], cuts[i + 1]) for i in range(d)]


def synthetic_remote_partials(batch, seed_offset=1000):
    """Timing-only stand-ins for partials other instances would push back (Phase 3):
    O ~ N(0, 0.02), LSE ~ N(log(range length), 0.5), float32.  Not comparable with exact attention."""
    rng = np.random.default_rng(batch.seed + seed_offset)
    n = len(batch.remote_meta)
    d = batch.desc
    o = (0.02 * rng.standard_normal((n, d.num_q_heads, d.head_dim_v))).astype(np.float32)
    lens = np.asarray([max(e - b, 1) for (_, _, b, e) in batch.remote_meta], np.float64).reshape(n, 1)
    lse = (np.log(lens) + 0.5 * rng.standard_normal((n, d.num_q_heads))).astype(np.float32)
    return o, lse
