"""Host side of the reduce-phase plan and of KV append (C ABI, no device): the integers
agree bit-exactly with the oracle's."""
import numpy as np
import pytest

import oracle
from paper_2605_06914_amd import Context, TaperError, append_slots, branch_blocks
from paper_2605_06914_amd import TAPER_EBLOCK, TAPER_EINVAL, TAPER_ELEN
from taper_inputs import AttnShape, reduce_structure, structure_custom

QWEN = AttnShape(64, 8, 128, 16)


def parallel_structure(seed=5, spare=60):
    reqs = [(37, [0]), (50, [0, 7, 16, 21]), (700, [0, 33, 64, 65, 129, 300]), (16, [1]), (333, list(range(20)))]
    st = structure_custom(QWEN, reqs, seed=seed)
    return structure_custom(QWEN, reqs, seed=seed, n_pool_pages=st.n_pool_pages + spare)


@pytest.mark.parametrize("keep", [(), (1, 4), (0, 1, 2, 3, 4)])
def test_segment_plan_integers_match_oracle(keep):
    par = parallel_structure()
    seg = reduce_structure(par, z_len=[5, 0, 40, 16, 200], seed=3, keep_parallel=keep)
    ctx = Context(64, 8, 128, device=-1)
    plan = ctx.plan_build_segments(seg.block_table, seg.branch_group, seg.prefix_len, seg.seg_start, seg.seg_len,
                                   seg.n_pool_pages)
    e = plan.export()
    ctx_len, npriv, slots = oracle.resolve_segments(16, seg.block_table, seg.prefix_len, seg.seg_start, seg.seg_len)
    assert np.array_equal(e["ctx_len"], ctx_len) and np.array_equal(e["n_suffix_pages"], npriv)
    assert np.array_equal(e["seg_start"], seg.seg_start) and np.array_equal(e["seg_len"], seg.seg_len)
    assert np.array_equal(plan.resolve_slots_host(slots.shape[1]), slots)
    assert e["tokens_logical"] == seg.logical_tokens
    # every logical position is covered by exactly one work item
    F = {n: i for i, n in enumerate(e["item_fields"])}
    cover = [np.zeros(int(c), np.int32) for c in ctx_len]
    page0_of = {}  # (sequence, block-table entry of a segment start) -> logical position
    for s in range(seg.n_seqs):
        pos, entry = int(seg.prefix_len[s]), -(-int(seg.prefix_len[s]) // 16)
        for k in range(seg.seg_start[s], seg.seg_start[s + 1]):
            for j in range(-(-int(seg.seg_len[k]) // 16)):
                page0_of[(s, entry + j)] = pos + 16 * j
            pos += int(seg.seg_len[k])
            entry += -(-int(seg.seg_len[k]) // 16)
    for it in e["items"]:
        seq0, nb, page0, ntok = (int(it[F[k]]) for k in ("seq0", "n_branch", "page0", "n_tokens"))
        for b in range(nb):
            s = seq0 + b
            lo = page0 * 16 if page0 * 16 < seg.prefix_len[s] else page0_of[(s, page0)]
            cover[s][lo : lo + ntok] += 1
    for s, c in enumerate(cover):
        assert np.all(c == 1), f"sequence {s} not covered exactly once"
    plan.free()


def test_segment_plan_rejects_malformed_input():
    par = parallel_structure()
    seg = reduce_structure(par, z_len=[5, 0, 40, 16, 200], seed=3)
    ctx = Context(64, 8, 128, device=-1)

    def build(**over):
        a = dict(block_table=seg.block_table, branch_group=seg.branch_group, prefix_len=seg.prefix_len,
                 seg_start=seg.seg_start.copy(), seg_len=seg.seg_len.copy(), n_pool_pages=seg.n_pool_pages)
        a.update(over)
        return ctx.plan_build_segments(**a)

    ss = seg.seg_start.copy()
    ss[0] = 1
    bad_len = seg.seg_len.copy()
    bad_len[2] = -4
    too_long = seg.seg_len.copy()
    too_long[-1] += 16 * 50  # needs pages the row does not list
    for over, code in ((dict(seg_start=ss), TAPER_EINVAL), (dict(seg_len=bad_len), TAPER_ELEN), (dict(seg_len=too_long), TAPER_ELEN)):
        with pytest.raises(TaperError) as e:
            build(**over)
        assert e.value.status == code
    dec = seg.seg_start.copy()
    dec[2] = dec[1] - 1
    with pytest.raises(TaperError):
        build(seg_start=dec)
    # a sequence whose segments are all empty and whose prefix is empty has no context
    with pytest.raises(TaperError) as e:
        ctx.plan_build_segments(np.zeros((1, 4), np.int32), [0], [0], [0, 2], [0, 0], 8)
    assert e.value.status == TAPER_ELEN


def test_append_slots_follow_the_last_segment():
    par = parallel_structure()
    seg = reduce_structure(par, z_len=[5, 0, 40, 16, 200], seed=3, keep_parallel=(1,))
    # give every row one spare entry holding a fresh page, for sequences whose last segment fills its pages
    bt = np.concatenate([seg.block_table, np.full((seg.n_seqs, 1), -1, np.int32)], axis=1)
    used = set(int(x) for x in bt.ravel() if x >= 0)
    fresh = [p for p in range(seg.n_pool_pages) if p not in used]
    want_slot, want_open = [], []
    for s in range(seg.n_seqs):
        lens = [int(x) for x in seg.seg_len[seg.seg_start[s]:seg.seg_start[s + 1]]]
        entry = -(-int(seg.prefix_len[s]) // 16) + sum(-(-n // 16) for n in lens[:-1]) + lens[-1] // 16
        if lens[-1] % 16 == 0:
            bt[s, entry] = fresh.pop()
        want_slot.append(int(bt[s, entry]) * 16 + lens[-1] % 16)
        want_open.append(int(lens[-1] % 16 == 0))
    slots, opens = append_slots(bt, seg.prefix_len, seg.seg_start, seg.seg_len, 16, seg.n_pool_pages)
    assert slots.tolist() == want_slot and opens.tolist() == want_open
    # the oracle resolves the appended token to the same slot once the segment has grown by one
    grown = seg.seg_len.copy()
    grown[seg.seg_start[1:] - 1] += 1
    ctx_len, _, oslots = oracle.resolve_segments(16, bt, seg.prefix_len, seg.seg_start, grown)
    assert [int(oslots[s, ctx_len[s] - 1]) for s in range(seg.n_seqs)] == want_slot
    # errors: no page entered for a token that opens a page; page outside the pool; nothing to append to
    missing = bt.copy()
    s_full = want_open.index(1)
    missing[s_full, np.flatnonzero(missing[s_full] >= 0)[-1]] = -1
    with pytest.raises(TaperError) as e:
        append_slots(missing, seg.prefix_len, seg.seg_start, seg.seg_len, 16, seg.n_pool_pages)
    assert e.value.status == TAPER_EBLOCK
    with pytest.raises(TaperError) as e:
        append_slots(seg.block_table[:, :2], seg.prefix_len, seg.seg_start, seg.seg_len, 16, seg.n_pool_pages)
    assert e.value.status == TAPER_ELEN
    with pytest.raises(TaperError) as e:
        append_slots(bt[:1], seg.prefix_len[:1], [0, 0], np.zeros(1, np.int32)[:0], 16, seg.n_pool_pages)
    assert e.value.status == TAPER_EINVAL


def test_branch_blocks_is_the_marginal_memory_of_a_branch():
    # App. C: blocks of the branch-local tokens; a branch that has produced nothing costs nothing
    assert [branch_blocks(n) for n in (0, 1, 15, 16, 17, 2048)] == [0, 1, 1, 1, 2, 128]
    par = parallel_structure()
    ints = oracle.resolve(16, par.block_table, par.branch_group, par.prefix_len, par.suffix_len, want_slots=False)
    assert [branch_blocks(int(n)) for n in par.suffix_len] == ints.n_suffix_pages.tolist()
