"""Seeded generators for decode-step batches with shared-prefix branches.

A *batch* is what a continuous-batching engine hands to one decode step
(paper §1, §2.3): S sequences, one new token each.  A sequence is either a
serial request or one admitted branch of a request in a parallel phase
(paper §3.1: phase = shared prefix + per-branch private tokens).  The branches
of one request reference a single set of prefix pages; each owns only its
private pages (paper §3.1, App. C "Memory accounting").

Everything here is integers and random values.  No attention arithmetic and
no in-page element layout lives in this module.

Draw order for every workload (one numpy PCG64 generator per workload):
serial contexts, prefix lengths, branch widths, suffix lengths, page
permutation; then (separate generator, seed+1000) q values, KV values.
"""
from __future__ import annotations

import dataclasses
import math
from typing import List, Optional, Sequence, Tuple

import numpy as np

CONFIG_SEED_BASE = 20260500
K = 1024


@dataclasses.dataclass(frozen=True)
class AttnShape:
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    page_size: int = 16

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.head_dim)

    @property
    def gqa(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def page_elems(self) -> int:
        """bf16 elements in one pool page (K and V, all KV heads)."""
        return 2 * self.n_kv_heads * self.page_size * self.head_dim

    @property
    def kv_bytes_per_token(self) -> int:
        return 2 * self.n_kv_heads * self.head_dim * 2


QWEN = AttnShape(64, 8, 128, 16)
TINY = AttnShape(4, 1, 64, 16)


@dataclasses.dataclass
class BatchStructure:
    """Integer side of a batch: who attends to which pages."""

    shape: AttnShape
    block_table: np.ndarray  # int32 [S, max_blocks]; unused entries are -1
    branch_group: np.ndarray  # int32 [S], non-decreasing request id
    prefix_len: np.ndarray  # int32 [S], equal inside a group
    suffix_len: np.ndarray  # int32 [S]
    n_pool_pages: int
    name: str = ""
    seed: int = 0

    @property
    def n_seqs(self) -> int:
        return int(self.block_table.shape[0])

    @property
    def n_groups(self) -> int:
        return int(self.branch_group[-1]) + 1 if self.n_seqs else 0

    @property
    def logical_tokens(self) -> int:
        return int(self.prefix_len.astype(np.int64).sum() + self.suffix_len.astype(np.int64).sum())

    @property
    def unique_tokens(self) -> int:
        first = np.ones(self.n_seqs, dtype=bool)
        first[1:] = self.branch_group[1:] != self.branch_group[:-1]
        return int(self.prefix_len[first].astype(np.int64).sum() + self.suffix_len.astype(np.int64).sum())

    @property
    def kv_bytes_unique(self) -> int:
        return self.unique_tokens * self.shape.kv_bytes_per_token

    @property
    def kv_bytes_logical(self) -> int:
        return self.logical_tokens * self.shape.kv_bytes_per_token

    @property
    def qo_bytes(self) -> int:
        return 2 * self.n_seqs * self.shape.n_q_heads * self.shape.head_dim * 2


@dataclasses.dataclass
class Batch:
    structure: BatchStructure
    q: np.ndarray  # uint16 (bf16 bits) [S, Hq, D]
    kv: np.ndarray  # uint16 (bf16 bits) [n_pool_pages, page_elems]


# ---------------------------------------------------------------- bf16 bits
def bf16_bits_from_f32(x: np.ndarray) -> np.ndarray:
    """Round float32 to the nearest bf16 (ties to even); returns uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def f32_from_bf16_bits(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ---------------------------------------------------------------- structure
Request = Tuple[int, Sequence[int]]  # (prefix_len, [suffix_len per admitted branch])


def build_structure(
    shape: AttnShape,
    requests: Sequence[Request],
    rng: np.random.Generator,
    pool_factor: float = 1.1,
    n_pool_pages: Optional[int] = None,
    reserve_branches: Optional[Sequence[Sequence[int]]] = None,
    name: str = "",
    seed: int = 0,
) -> BatchStructure:
    """Lay the requests out over a randomly permuted page pool.

    Pages are handed out in logical order (request by request: prefix pages,
    then each branch's private pages) from one random permutation of the pool,
    so neighbours in a block table are scattered in memory.  A branch's
    private tokens start on a fresh page even when the prefix ends mid-page.

    ``reserve_branches[r]`` may list suffix lengths of *all* branches of
    request r (a superset of the admitted ones, admitted = its first entries):
    pages are then drawn for every listed branch, so the admitted branches keep
    the same pages whatever the admitted count is.
    """
    P = shape.page_size
    cdiv = lambda a: (int(a) + P - 1) // P
    alloc: List[Sequence[int]] = []
    for r, (_, suf) in enumerate(requests):
        full = list(reserve_branches[r]) if reserve_branches is not None else list(suf)
        assert list(full[: len(suf)]) == list(suf)
        alloc.append(full)
    used = sum(cdiv(p) + sum(cdiv(s) for s in alloc[r]) for r, (p, _) in enumerate(requests))
    if n_pool_pages is None:
        n_pool_pages = max(1, int(math.ceil(pool_factor * used)))
    assert used <= n_pool_pages, (used, n_pool_pages)
    if n_pool_pages > 4 * used + 1024:
        # large sparse pool: draw distinct page ids without a full permutation
        pages = rng.choice(n_pool_pages, size=used, replace=False).astype(np.int64)
    else:
        pages = rng.permutation(n_pool_pages)[:used].astype(np.int64)
    n_seqs = sum(len(suf) for _, suf in requests)
    max_blocks = max([cdiv(p) + max([cdiv(s) for s in suf] + [0]) for p, suf in requests] + [1])
    bt = np.full((n_seqs, max_blocks), -1, dtype=np.int32)
    grp = np.zeros(n_seqs, dtype=np.int32)
    pl = np.zeros(n_seqs, dtype=np.int32)
    sl = np.zeros(n_seqs, dtype=np.int32)
    cur = 0
    s = 0
    for r, (p, suf) in enumerate(requests):
        npp = cdiv(p)
        ppages = pages[cur : cur + npp]
        cur += npp
        for b, sfx in enumerate(alloc[r]):
            nsp = cdiv(sfx)
            spages = pages[cur : cur + nsp]
            cur += nsp
            if b < len(suf):
                bt[s, :npp] = ppages
                bt[s, npp : npp + nsp] = spages
                grp[s] = r
                pl[s] = p
                sl[s] = sfx
                s += 1
    assert s == n_seqs and cur == used
    return BatchStructure(shape, bt, grp, pl, sl, int(n_pool_pages), name=name, seed=seed)


def structure_custom(shape, requests, seed=0, **kw) -> BatchStructure:
    return build_structure(shape, requests, np.random.default_rng(np.random.PCG64(seed)), seed=seed, **kw)


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def structure_config1(seed: int = CONFIG_SEED_BASE + 1) -> BatchStructure:
    """Tiny: one serial request (256) + one request with prefix 192 and 4
    branches with private suffixes 0, 8, 17, 32, in a 64-page pool."""
    reqs = [(256, [0]), (192, [0, 8, 17, 32])]
    return build_structure(TINY, reqs, _rng(seed), n_pool_pages=64, name="config1_tiny", seed=seed)


def structure_config2(seed: int = CONFIG_SEED_BASE + 2, n_serial: int = 32) -> BatchStructure:
    """IRP-Off shape: 32 serial requests, contexts uniform on [1024, 4096]."""
    rng = _rng(seed)
    ctx = rng.integers(1 * K, 4 * K, size=n_serial, endpoint=True)
    reqs = [(int(c), [0]) for c in ctx]
    return build_structure(QWEN, reqs, rng, pool_factor=1.1, name="config2_irp_off", seed=seed)


def structure_config3(seed: int = CONFIG_SEED_BASE + 3) -> BatchStructure:
    """Mixed: 16 serial (1k-4k) + 8 parallel requests, prefix 2k-8k, width
    4-8, private suffix 0-1024."""
    rng = _rng(seed)
    ctx = rng.integers(1 * K, 4 * K, size=16, endpoint=True)
    pre = rng.integers(2 * K, 8 * K, size=8, endpoint=True)
    wid = rng.integers(4, 8, size=8, endpoint=True)
    suf = [rng.integers(0, 1 * K, size=int(w), endpoint=True) for w in wid]
    reqs = [(int(c), [0]) for c in ctx] + [(int(p), [int(x) for x in s]) for p, s in zip(pre, suf)]
    return build_structure(QWEN, reqs, rng, pool_factor=1.1, name="config3_mixed", seed=seed)


def structure_config4(seed: int = CONFIG_SEED_BASE + 4, pool_bytes: float = 30e9) -> BatchStructure:
    """Long context: 32 serial (1k-8k) + 8 requests with a 32768-token prefix
    and 16 branches (suffix 0-2048); used pages scattered in a ~30 GB pool."""
    rng = _rng(seed)
    ctx = rng.integers(1 * K, 8 * K, size=32, endpoint=True)
    suf = [rng.integers(0, 2 * K, size=16, endpoint=True) for _ in range(8)]
    reqs = [(int(c), [0]) for c in ctx] + [(32 * K, [int(x) for x in s]) for s in suf]
    n_pool = int(pool_bytes // (QWEN.page_elems * 2))
    return build_structure(QWEN, reqs, rng, n_pool_pages=n_pool, name="config4_long", seed=seed)


def structure_config5(k: int, seed: int = CONFIG_SEED_BASE + 5, n_serial: int = 96, n_parallel: int = 32,
                      fanout: int = 17) -> BatchStructure:
    """Admission sweep, one layer's structure: 96 serial (512-8k) + 32 parallel
    requests (prefix 1k-16k, suffix 0-2k).  Each parallel request runs its
    protected branch plus k opportunistic ones (paper §2.3, §3.3): width 1+k.
    The 17 branches per request are drawn once; k selects a nested prefix of
    them and every branch keeps its pages for every k."""
    assert 0 <= k <= fanout - 1
    rng = _rng(seed)
    ctx = rng.integers(512, 8 * K, size=n_serial, endpoint=True)
    pre = rng.integers(1 * K, 16 * K, size=n_parallel, endpoint=True)
    suf = [[int(x) for x in rng.integers(0, 2 * K, size=fanout, endpoint=True)] for _ in range(n_parallel)]
    reqs = [(int(c), [0]) for c in ctx] + [(int(p), s[: 1 + k]) for p, s in zip(pre, suf)]
    reserve = [[0] for _ in ctx] + suf
    return build_structure(QWEN, reqs, rng, pool_factor=1.1, reserve_branches=reserve,
                           name=f"config5_sweep_k{k}", seed=seed)


def structure_wide(width: int, seed: int = CONFIG_SEED_BASE + 6) -> BatchStructure:
    """Wide requests: the mixed batch's shape (16 serial 1k-4k, 8 parallel with prefix 2k-8k and
    private suffix 0-1024) with every parallel request at `width` branches -- wider than one
    workgroup's row tiles hold, so a prefix is listed for more than one group of branches."""
    rng = _rng(seed)
    ctx = rng.integers(1 * K, 4 * K, size=16, endpoint=True)
    pre = rng.integers(2 * K, 8 * K, size=8, endpoint=True)
    suf = [rng.integers(0, 1 * K, size=width, endpoint=True) for _ in range(8)]
    reqs = [(int(c), [0]) for c in ctx] + [(int(p), [int(x) for x in s]) for p, s in zip(pre, suf)]
    return build_structure(QWEN, reqs, rng, pool_factor=1.1, name=f"wide_requests_w{width}", seed=seed)


def make_config(index: int, **kw) -> BatchStructure:
    return {1: structure_config1, 2: structure_config2, 3: structure_config3,
            4: structure_config4, 5: structure_config5}[index](**kw)


# ---------------------------------------------------------------- values
def fill_values_numpy(st: BatchStructure, seed: Optional[int] = None, chunk_pages: int = 4096) -> Batch:
    """i.i.d. N(0,1) values rounded to bf16 for q and for every pool page
    (referenced or not).  Host memory: 2 B per element; meant for pools up to
    a few GB."""
    seed = (st.seed + 1000) if seed is None else seed
    rng = _rng(seed)
    sh = st.shape
    q = bf16_bits_from_f32(rng.standard_normal((st.n_seqs, sh.n_q_heads, sh.head_dim), dtype=np.float32))
    kv = np.empty((st.n_pool_pages, sh.page_elems), dtype=np.uint16)
    for p0 in range(0, st.n_pool_pages, chunk_pages):
        p1 = min(st.n_pool_pages, p0 + chunk_pages)
        kv[p0:p1] = bf16_bits_from_f32(rng.standard_normal((p1 - p0, sh.page_elems), dtype=np.float32))
    return Batch(st, q, kv)


def subset_rows(st: BatchStructure, seq_ids: Sequence[int]) -> BatchStructure:
    """The sequences ``seq_ids`` (ascending) over the SAME pool: rows of the block table are kept as they
    are, group ids are renumbered densely (a group keeps its sharing)."""
    seq_ids = np.asarray(seq_ids, dtype=np.int64)
    assert len(seq_ids) and np.all(np.diff(seq_ids) > 0)
    g_old = st.branch_group[seq_ids]
    g_new = np.zeros(len(seq_ids), dtype=np.int32)
    g_new[1:] = np.cumsum(g_old[1:] != g_old[:-1])
    return BatchStructure(st.shape, np.ascontiguousarray(st.block_table[seq_ids]), g_new, st.prefix_len[seq_ids].copy(),
                          st.suffix_len[seq_ids].copy(), st.n_pool_pages, name=st.name + "_subset", seed=st.seed)


def compact_rows(st: BatchStructure, seq_ids: Sequence[int]) -> Tuple[BatchStructure, np.ndarray]:
    """Sub-batch holding only ``seq_ids`` (ascending), over a compact pool.

    Returns the new structure and the int64 array ``page_ids`` such that new
    pool page i is old pool page ``page_ids[i]`` (gather the KV rows with it).
    Group ids are renumbered densely; a group keeps its sharing."""
    seq_ids = np.asarray(seq_ids, dtype=np.int64)
    assert np.all(np.diff(seq_ids) > 0)
    P = st.shape.page_size
    bt_old = st.block_table[seq_ids]
    pl = st.prefix_len[seq_ids].copy()
    sl = st.suffix_len[seq_ids].copy()
    npages = (pl + P - 1) // P + (sl + P - 1) // P
    remap = {}
    order: List[int] = []
    bt_new = np.full_like(bt_old, -1)
    for i in range(len(seq_ids)):
        for j in range(int(npages[i])):
            pg = int(bt_old[i, j])
            if pg not in remap:
                remap[pg] = len(order)
                order.append(pg)
            bt_new[i, j] = remap[pg]
    g_old = st.branch_group[seq_ids]
    g_new = np.zeros(len(seq_ids), dtype=np.int32)
    if len(seq_ids):
        g_new[1:] = np.cumsum(g_old[1:] != g_old[:-1])
    sub = BatchStructure(st.shape, bt_new, g_new, pl, sl, max(1, len(order)), name=st.name + "_sub", seed=st.seed)
    return sub, np.asarray(order, dtype=np.int64)


# ---------------------------------------------------------------- segmented contexts (reduce phase)
@dataclasses.dataclass
class SegmentedStructure:
    """A batch whose sequences see the shared prefix followed by a LIST of private segments, each written on
    pages of its own (paper §3.1: a branch sees one private segment, h_i ++ y_i so far; a reduce token sees
    every completed branch in canonical order and then the reduce tokens so far)."""

    shape: AttnShape
    block_table: np.ndarray  # int32 [S, max_blocks]: prefix pages, then each segment's pages in order
    branch_group: np.ndarray  # int32 [S]
    prefix_len: np.ndarray  # int32 [S], equal inside a group
    seg_start: np.ndarray  # int32 [S + 1] CSR over seg_len
    seg_len: np.ndarray  # int32, tokens of each private segment (may be 0: owns no page)
    n_pool_pages: int
    name: str = ""
    seed: int = 0

    @property
    def n_seqs(self) -> int:
        return int(self.block_table.shape[0])

    @property
    def private_len(self) -> np.ndarray:
        return np.array([int(self.seg_len[self.seg_start[s]:self.seg_start[s + 1]].sum()) for s in range(self.n_seqs)],
                        dtype=np.int64)

    @property
    def logical_tokens(self) -> int:
        return int(self.prefix_len.astype(np.int64).sum() + self.private_len.sum())


def reduce_structure(par: BatchStructure, z_len: Sequence[int], seed: int = 0, keep_parallel: Sequence[int] = ()) -> SegmentedStructure:
    """The step after a parallel phase.  Every request (group) of ``par`` not listed in ``keep_parallel``
    becomes ONE reduce sequence: its prefix pages, then the private pages of each of its branches in branch
    order (the pages ``par`` gave them, partially filled last pages included), then ``z_len[g]`` reduce tokens
    on fresh pages taken from the pool's unused pages.  Requests in ``keep_parallel`` stay as they are
    (branches with one private segment each), so both phases can share a batch."""
    P = par.shape.page_size
    cdiv = lambda a: (int(a) + P - 1) // P
    rng = np.random.Generator(np.random.PCG64(seed))
    used = np.zeros(par.n_pool_pages, dtype=bool)
    for s in range(par.n_seqs):
        n = cdiv(par.prefix_len[s]) + cdiv(par.suffix_len[s])
        used[par.block_table[s, :n]] = True
    free = rng.permutation(np.flatnonzero(~used))
    rows, grp, pl, segs = [], [], [], []
    cur = 0
    g_new = 0
    first = np.flatnonzero(np.r_[True, par.branch_group[1:] != par.branch_group[:-1]])
    bounds = np.r_[first, par.n_seqs]
    for g in range(par.n_groups):
        a, b = int(bounds[g]), int(bounds[g + 1])
        npp = cdiv(par.prefix_len[a])
        if g in keep_parallel:
            for s in range(a, b):
                rows.append(list(par.block_table[s, : npp + cdiv(par.suffix_len[s])]))
                grp.append(g_new)
                pl.append(int(par.prefix_len[s]))
                segs.append([int(par.suffix_len[s])])
        else:
            row = list(par.block_table[a, :npp])
            seg = []
            for s in range(a, b):
                row += list(par.block_table[s, npp : npp + cdiv(par.suffix_len[s])])
                seg.append(int(par.suffix_len[s]))
            nz = cdiv(z_len[g])
            assert cur + nz <= len(free), "pool has too few unused pages for the reduce tokens"
            row += list(free[cur : cur + nz])
            cur += nz
            seg.append(int(z_len[g]))
            rows.append(row)
            grp.append(g_new)
            pl.append(int(par.prefix_len[a]))
            segs.append(seg)
        g_new += 1
    width = max(len(r) for r in rows)
    bt = np.full((len(rows), max(width, 1)), -1, dtype=np.int32)
    for i, r in enumerate(rows):
        bt[i, : len(r)] = r
    seg_start = np.zeros(len(rows) + 1, dtype=np.int32)
    seg_start[1:] = np.cumsum([len(x) for x in segs])
    seg_len = np.array([v for x in segs for v in x], dtype=np.int32)
    return SegmentedStructure(par.shape, bt, np.array(grp, np.int32), np.array(pl, np.int32), seg_start, seg_len,
                              par.n_pool_pages, name=par.name + "_reduce", seed=seed)
