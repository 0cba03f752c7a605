"""CPU-only tests of the C-ABI library: it loads, exports every declared symbol,
validates its inputs, and its integer plan agrees bit-exactly with the oracle's
integer side.  No device call is made (host-only contexts)."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_2605_06914_amd import (Context, EXPORTED, LIB_PATH, TaperError, load_library, TAPER_EBLOCK, TAPER_EGROUP,
                                  TAPER_EHIP, TAPER_EINVAL, TAPER_ELEN)
from taper_inputs import (AttnShape, structure_config1, structure_config2, structure_config3, structure_config4,
                          structure_config5, structure_custom)

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
QWEN = AttnShape(64, 8, 128, 16)


def test_library_exports_every_declared_symbol():
    lib = load_library()
    header = "".join(open(os.path.join(ROOT, "include", f)).read() for f in sorted(os.listdir(os.path.join(ROOT, "include"))))
    declared = set(re.findall(r"TAPER_API\s+[\w\s\*]+?\b(taper_\w+)\s*\(", header))
    assert declared == set(EXPORTED), declared ^ set(EXPORTED)
    for name in declared:
        assert getattr(lib, name) is not None
    assert os.path.exists(LIB_PATH)
    assert lib.taper_strerror(-3) == b"malformed request grouping"


def host_ctx(sh=QWEN):
    return Context(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.page_size, device=-1)


def build(st, ctx=None, **kw):
    ctx = ctx or host_ctx(st.shape)
    return ctx.plan_build(st.block_table, st.branch_group, st.prefix_len, st.suffix_len, st.n_pool_pages, **kw)


@pytest.mark.parametrize("bad", [dict(n_q_heads=64, n_kv_heads=7), dict(head_dim=96), dict(page_size=32),
                                 dict(n_q_heads=64, n_kv_heads=2), dict(scale=0.0)])
def test_create_rejects_unsupported_shapes(bad):
    kw = dict(n_q_heads=64, n_kv_heads=8, head_dim=128, page_size=16, scale=None, device=-1)
    kw.update(bad)
    with pytest.raises(TaperError) as e:
        Context(**kw)
    assert e.value.status == TAPER_EINVAL


def test_validation_errors():
    st = structure_config1()
    ctx = host_ctx(st.shape)

    def expect(code, **over):
        args = dict(block_table=st.block_table.copy(), branch_group=st.branch_group.copy(),
                    prefix_len=st.prefix_len.copy(), suffix_len=st.suffix_len.copy(), n_pool_pages=st.n_pool_pages)
        for k, f in over.items():
            args[k] = f(args[k])
        with pytest.raises(TaperError) as e:
            ctx.plan_build(**args)
        assert e.value.status == code, (e.value, code)

    def setv(i, v):
        def f(a):
            a = a.copy()
            a[i] = v
            return a
        return f

    expect(TAPER_EBLOCK, block_table=setv((0, 3), -1))
    expect(TAPER_EBLOCK, block_table=setv((4, 13), 64))
    expect(TAPER_EBLOCK, n_pool_pages=lambda n: 10)
    expect(TAPER_EGROUP, branch_group=setv(0, 1))
    expect(TAPER_EGROUP, branch_group=setv(2, 3))
    expect(TAPER_EGROUP, branch_group=lambda a: np.array([0, 1, 1, 0, 1], np.int32))
    expect(TAPER_EGROUP, prefix_len=setv(3, 191))
    expect(TAPER_EGROUP, block_table=setv((2, 5), int(st.block_table[0, 0])))  # a member's prefix page differs
    expect(TAPER_ELEN, suffix_len=setv(2, -1))
    expect(TAPER_ELEN, prefix_len=lambda a: np.array([0, 192, 192, 192, 192], np.int32))  # serial request left empty
    expect(TAPER_ELEN, suffix_len=setv(4, 16 * 10))  # row too short for its pages
    expect(TAPER_EINVAL, n_pool_pages=lambda n: 0)
    # unused block-table entries may hold anything
    bt = st.block_table.copy()
    bt[bt < 0] = 123456
    ctx.plan_build(bt, st.branch_group, st.prefix_len, st.suffix_len, st.n_pool_pages).free()


def test_host_only_context_refuses_device_work():
    st = structure_config1()
    ctx = host_ctx(st.shape)
    plan = build(st, ctx)
    with pytest.raises(TaperError) as e:
        load = load_library()
        rc = load.taper_decode_step_attention(ctx._h, plan._h, 8, 8, 8, None, None)
        if rc != 0:
            raise TaperError(rc, load.taper_last_error().decode())
    assert e.value.status == TAPER_EHIP


def check_plan_against_oracle(st, **kw):
    sh = st.shape
    g = sh.gqa
    plan = build(st, **kw)
    e = plan.export()
    ints = oracle.resolve(sh.page_size, st.block_table, st.branch_group, st.prefix_len, st.suffix_len,
                          want_slots=st.logical_tokens < 2_000_000)
    assert e["n_groups"] == ints.n_groups and e["n_seqs"] == st.n_seqs
    for key in ("ctx_len", "n_prefix_pages", "n_suffix_pages", "group_start"):
        assert np.array_equal(e[key], getattr(ints, key)), key
    assert e["tokens_unique"] == st.unique_tokens and e["tokens_logical"] == st.logical_tokens
    if ints.slots is not None:
        assert np.array_equal(plan.resolve_slots_host(ints.slots.shape[1]), ints.slots)
    # every (sequence, logical position) is covered by exactly one work item
    F = {n: i for i, n in enumerate(e["item_fields"])}
    items = e["items"]
    cover = [np.zeros(int(c), np.int32) for c in ints.ctx_len]
    for it in items:
        seq0, nb, page0, ntok, kind = (int(it[F[k]]) for k in ("seq0", "n_branch", "page0", "n_tokens", "kind"))
        assert ntok >= 1 and nb >= 1 and (kind == 0) == (nb >= 2)
        assert nb * g <= 12 * 16
        npp = int(ints.n_prefix_pages[seq0])
        for b in range(nb):
            s = seq0 + b
            assert st.branch_group[s] == st.branch_group[seq0]
            if page0 < npp or ints.n_suffix_pages[seq0] == 0 and st.suffix_len[seq0] == 0:
                lo = page0 * 16  # inside the prefix
                assert lo + ntok <= st.prefix_len[s]
            else:
                assert nb == 1
                lo = int(st.prefix_len[s]) + (page0 - npp) * 16
            cover[s][lo : lo + ntok] += 1
    for s, c in enumerate(cover):
        assert np.all(c == 1), f"sequence {s} not covered exactly once"
    # parts partition the items; partial rows are disjoint; merge map lists each sequence's items
    # after them the pool: private items that belong to no share
    ps = e["part_start"]
    n_pool = e["n_pool_items"]
    assert ps[0] == 0 and ps[-1] + n_pool == len(items) and np.all(np.diff(ps) >= 1)
    assert np.array_equal(items[: ps[-1], F["part"]], np.repeat(np.arange(len(ps) - 1), np.diff(ps)))
    assert np.all(items[ps[-1] :, F["part"]] == len(ps) - 1) and np.all(items[ps[-1] :, F["n_branch"]] == 1)
    pool_cap = max(32, (kw.get("pool_item_tokens", 0) or 1536) // 32 * 32)
    assert np.all(items[ps[-1] :, F["n_tokens"]] <= pool_cap)
    nsh = e["n_parts_shared"]
    assert np.all(items[: ps[nsh], F["kind"]] == 0) and np.all(items[ps[nsh] :, F["kind"]] >= 1)
    rows = items[:, F["n_branch"]].astype(np.int64) * g * sh.n_kv_heads
    assert np.array_equal(items[:, F["part_base"]], np.concatenate([[0], np.cumsum(rows)[:-1]]))
    assert e["n_partial_rows"] == rows.sum()
    ms, merge = e["merge_start"], e["merge"]
    for s in range(st.n_seqs):
        its = [it for it in items if it[F["seq0"]] <= s < it[F["seq0"]] + it[F["n_branch"]]]
        mine = [(int(it[F["part_base"]]) + (s - int(it[F["seq0"]])) * g, int(it[F["n_branch"]]) * g) for it in its]
        assert [tuple(x) for x in merge[ms[s] : ms[s + 1]]] == mine
        # kind 2 marks exactly the private items that are their sequence's only item
        assert all((int(it[F["kind"]]) >= 2) == (len(its) == 1 and it[F["n_branch"]] == 1) for it in its)
    plan.free()
    return e


@pytest.mark.parametrize("maker", [structure_config1, structure_config2, structure_config3,
                                   lambda: structure_config5(k=16, n_serial=12, n_parallel=5)])
def test_plan_integers_match_oracle(maker):
    check_plan_against_oracle(maker())


@pytest.mark.parametrize("kw", [dict(share_prefix=False), dict(target_workgroups=8), dict(target_workgroups=100000), dict(target_workgroups=100000, min_share_tokens=1),
                                dict(max_branches_per_item=3), dict(scatter_sub_groups=True), dict(max_branches_per_item=4, scatter_sub_groups=True), dict(pool_pct=-1), dict(pool_pct=90, pool_item_tokens=64), dict(pool_pct=100, pool_item_tokens=200),
                                dict(shared_cost_pct=300, shared_item_cost=5000, private_item_cost=1)])
def test_plan_options(kw):
    reqs = [(37, [0]), (50, [0, 7, 16, 21]), (16, [1]), (700, [0, 33, 64, 65, 129, 300]), (1, [0]), (0, [45]),
            (333, list(range(30)))]
    e = check_plan_against_oracle(structure_custom(QWEN, reqs, seed=1), **kw)
    if kw.get("share_prefix") is False:
        assert e["n_parts_shared"] == 0
    if kw.get("pool_pct") == -1:
        assert e["n_pool_items"] == 0
    if kw.get("pool_pct") == 90:
        F = {n: i for i, n in enumerate(e["item_fields"])}
        it = e["items"]
        priv = it[it[:, F["kind"]] >= 1]
        pooled = it[e["part_start"][-1] :, F["n_tokens"]].sum()
        assert 0.85 * priv[:, F["n_tokens"]].sum() <= pooled <= 0.9 * priv[:, F["n_tokens"]].sum() + 64


def test_config4_plan_is_balanced():
    st = structure_config4()
    e = check_plan_against_oracle(st)
    F = {n: i for i, n in enumerate(e["item_fields"])}
    ps = e["part_start"]
    tok = np.array([e["items"][ps[i] : ps[i + 1], F["n_tokens"]].sum() for i in range(len(ps) - 1)])
    nsh = e["n_parts_shared"]
    assert nsh > 0 and (nsh + e["n_parts_private"]) * 8 <= 600
    for t in (tok[:nsh], tok[nsh:]):
        assert t.max() <= 1.25 * t.sum() / len(t) + 64


@pytest.mark.parametrize("width,target", [(32, 0), (64, 0), (64, 4096), (100, 64)])
def test_sub_groups_of_a_wide_request_stream_the_prefix_side_by_side(width, target):
    """A request wider than one item is cut into sub-groups that each read the whole prefix.  Their items
    have the same cuts, a share each, and neighbouring shares (workgroups that start together and, for one
    kv head, sit on one XCD), chunk by chunk; with scatter_sub_groups they are placed like unrelated requests."""
    from taper_inputs import structure_wide

    st = structure_wide(width) if width <= 64 else structure_custom(QWEN, [(900, [0]), (5000, [7] * width), (70, [1, 2])], seed=3)
    e = check_plan_against_oracle(st, target_workgroups=target)
    F = {n: i for i, n in enumerate(e["item_fields"])}
    items, ps = e["items"], e["part_start"]
    shared = items[items[:, F["kind"]] == 0]
    sizes = np.bincount(st.branch_group)
    first = np.concatenate([[0], np.cumsum(sizes)[:-1]])
    checked = 0
    for g in np.flatnonzero(sizes > 24):
        mine = shared[(shared[:, F["seq0"]] >= first[g]) & (shared[:, F["seq0"]] < first[g] + sizes[g])]
        n_sub = -(-int(sizes[g]) // 24)
        assert len(mine) % n_sub == 0 and len(np.unique(mine[:, F["seq0"]])) == n_sub
        parts = mine[:, F["part"]]
        assert np.array_equal(parts, parts[0] + np.arange(len(mine))), "neighbouring shares, in order"
        assert np.all(np.diff(ps)[parts] == 1), "a share each"
        for c in range(len(mine) // n_sub):  # chunk c of every sub-group: the same pages
            chunk = mine[c * n_sub : (c + 1) * n_sub]
            assert len(set(chunk[:, F["page0"]])) == 1 and len(set(chunk[:, F["n_tokens"]])) == 1
            assert sorted(chunk[:, F["seq0"]]) == sorted(np.unique(mine[:, F["seq0"]]))
        checked += 1
    assert checked >= 1


def test_small_steps_without_shared_work_take_half_the_grid_when_that_saves_pieces():
    """With the grid left to the library, a step of serial requests is cut for one workgroup per compute unit
    instead of two when that cuts sequences into so many fewer pieces that it pays; never with shared-prefix
    work, never for an explicit grid (unless asked), never when nothing is saved; the plan is a full cover
    either way."""
    F = None

    def pieces(e):
        nonlocal F
        F = {n: i for i, n in enumerate(e["item_fields"])}
        return int((e["items"][:, F["kind"]] == 1).sum())

    irp = structure_config2()
    auto, never, explicit = (check_plan_against_oracle(irp, **kw) for kw in ({}, dict(small_step_grid=-1), dict(target_workgroups=512)))
    assert never["n_parts_private"] == explicit["n_parts_private"] == 64 and auto["n_parts_private"] == 32
    assert pieces(auto) < pieces(never) == pieces(explicit)
    asked = check_plan_against_oracle(irp, target_workgroups=512, small_step_grid=1)
    assert asked["n_parts_private"] == 32
    equal = structure_custom(QWEN, [(1024, [0])] * 32, seed=1)  # 256 (sequence, kv head) pairs: a workgroup each, nothing cut
    e = check_plan_against_oracle(equal)
    assert e["n_parts_private"] == 32 and pieces(e) == 0
    uncut = structure_custom(QWEN, [(1024, [0])] * 128, seed=1)  # nothing is cut at the full grid: nothing to save
    assert check_plan_against_oracle(uncut)["n_parts_private"] == 64
    big = structure_config5(k=0)  # long shares: the pieces saved do not pay for the slower grid
    assert check_plan_against_oracle(big)["n_parts_private"] == 64
    mixed = check_plan_against_oracle(structure_config3())
    assert mixed["n_parts_shared"] + mixed["n_parts_private"] == 64
