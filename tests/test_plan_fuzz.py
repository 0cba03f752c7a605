"""Seeded random batches and plan options through the host planner (C ABI, no device).

What the kernels assume of a plan is checked against the oracle's slot lists: every work
item reads, for every branch it serves, a run of physical slots that is exactly a run of
that sequence's logical positions (so no item crosses a half-filled page), the runs of a
sequence tile its context exactly once, and every index the kernels form from the plan
(partial rows, merge lists, pages) is in bounds.
"""
import numpy as np
import pytest

import oracle
from paper_2605_06914_amd import Context
from taper_inputs import AttnShape, reduce_structure, structure_custom

QWEN = AttnShape(64, 8, 128, 16)
TINY = AttnShape(4, 1, 64, 16)


def random_case(seed, shape):
    rng = np.random.default_rng(7000 + seed)
    reqs = []
    for _ in range(int(rng.integers(1, 24))):
        kind = rng.integers(0, 4)
        if kind == 0:
            reqs.append((int(rng.integers(1, 400)), [0]))
        elif kind == 1:
            reqs.append((0, [int(rng.integers(1, 6000))]))
        else:
            width = int(rng.choice([2, 3, 4, 7, 8, 9, 15, 16, 17, 24, 33]))
            suf = rng.integers(0, 300, size=width) * rng.integers(0, 2, size=width)
            reqs.append((int(rng.integers(1, 4000)), [int(x) for x in suf]))
    st = structure_custom(shape, reqs, seed=8000 + seed)
    st = structure_custom(shape, reqs, seed=8000 + seed, n_pool_pages=st.n_pool_pages + 80)
    n_groups = int(st.branch_group[-1]) + 1
    keep = [g for g in range(n_groups) if rng.random() < 0.5]
    seg = reduce_structure(st, z_len=[int(x) for x in rng.integers(0, 70, size=n_groups)], seed=seed, keep_parallel=keep)
    opts = {}
    if rng.random() < 0.6:
        opts["target_workgroups"] = int(rng.choice([1, 8, 64, 512, 4096, 100000]))
    if rng.random() < 0.5:
        opts["pool_pct"] = int(rng.choice([-1, 10, 50, 90]))
    if rng.random() < 0.3:
        opts["pool_item_tokens"] = int(rng.choice([32, 100, 512, 5000]))
    if rng.random() < 0.4:
        opts["min_share_tokens"] = int(rng.choice([1, 64, 1000, 100000]))
    if rng.random() < 0.3:
        opts["solo_item_tokens"] = int(rng.choice([-1, 32, 4096]))
    if rng.random() < 0.3:
        opts["max_branches_per_item"] = int(rng.choice([2, 5, 16, 24]))
    if rng.random() < 0.3:
        opts["shared_cost_pct"] = int(rng.choice([100, 400]))
        opts["shared_item_cost"] = int(rng.choice([1, 5000]))
    if rng.random() < 0.2:
        opts["share_prefix"] = 0
    if rng.random() < 0.25:
        opts["scatter_sub_groups"] = 1
    return seg, opts


@pytest.mark.parametrize("seed", range(48))
def test_random_plans_are_exact_covers_with_in_bounds_indices(seed):
    shape = TINY if seed % 6 == 5 else QWEN
    seg, opts = random_case(seed, shape)
    g = shape.gqa
    ctx = Context(shape.n_q_heads, shape.n_kv_heads, shape.head_dim, device=-1)
    plan = ctx.plan_build_segments(seg.block_table, seg.branch_group, seg.prefix_len, seg.seg_start, seg.seg_len,
                                   seg.n_pool_pages, **opts)
    e = plan.export()
    ctx_len, _, slots = oracle.resolve_segments(16, seg.block_table, seg.prefix_len, seg.seg_start, seg.seg_len)
    assert np.array_equal(e["ctx_len"], ctx_len)
    assert np.array_equal(plan.resolve_slots_host(slots.shape[1]), slots)
    F = {n: i for i, n in enumerate(e["item_fields"])}
    items = e["items"]
    bt = np.asarray(seg.block_table)
    where = [{int(v): i for i, v in enumerate(slots[s, : ctx_len[s]])} for s in range(seg.n_seqs)]
    cover = [np.zeros(int(c), np.int32) for c in ctx_len]
    # default: 12 tiles of 16 rows per item at head_dim 128, 8 at 64; an option may set up to 12
    cap = min(opts.get("max_branches_per_item", 0) or (12 if shape.head_dim == 128 else 8) * 16 // g, 12 * 16 // g)
    for it in items:
        seq0, nb, page0, ntok, kind, base = (int(it[F[k]]) for k in ("seq0", "n_branch", "page0", "n_tokens", "kind", "part_base"))
        assert 1 <= nb <= cap and ntok >= 1
        assert (kind == 0) == (nb >= 2) and 0 <= seq0 and seq0 + nb <= seg.n_seqs
        assert 0 <= base and base + nb * g * shape.n_kv_heads <= e["n_partial_rows"]
        n_pages = -(-ntok // 16)
        assert page0 + n_pages <= bt.shape[1]
        for b in range(nb):
            s = seq0 + b
            pages = bt[s, page0 : page0 + n_pages].astype(np.int64)
            assert np.all((0 <= pages) & (pages < seg.n_pool_pages))
            phys = (pages[:, None] * 16 + np.arange(16)[None, :]).reshape(-1)[:ntok]
            lo = where[s].get(int(phys[0]))
            assert lo is not None, "item starts at a slot the sequence does not own"
            assert lo + ntok <= ctx_len[s] and np.array_equal(slots[s, lo : lo + ntok], phys)
            cover[s][lo : lo + ntok] += 1
    for s, c in enumerate(cover):
        assert np.all(c == 1), f"sequence {s} not covered exactly once"
    # the parts tile the item list; the pool follows them
    ps = e["part_start"]
    assert ps[0] == 0 and np.all(np.diff(ps) >= 1) and ps[-1] + e["n_pool_items"] == len(items)
    assert len(ps) - 1 == e["n_parts_shared"] + e["n_parts_private"]
    # merge lists name each sequence's partial rows, inside the partial buffer
    ms, merge = e["merge_start"], e["merge"]
    assert ms[0] == 0 and ms[-1] == len(merge) and len(ms) == seg.n_seqs + 1
    for s in range(seg.n_seqs):
        its = [it for it in items if it[F["seq0"]] <= s < it[F["seq0"]] + it[F["n_branch"]]]
        mine = [(int(it[F["part_base"]]) + (s - int(it[F["seq0"]])) * g, int(it[F["n_branch"]]) * g) for it in its]
        assert [tuple(x) for x in merge[ms[s] : ms[s + 1]]] == mine
        assert all((int(it[F["kind"]]) >= 2) == (len(its) == 1 and it[F["n_branch"]] == 1) for it in its)
    plan.free()
    ctx.close()
