"""GPU tests of what surrounds the arithmetic: workspace lifetime under captured graphs, stale
partial rows of an earlier batch, both partial formats, and values of V far beyond the
half-precision range.  All through the C ABI, all against the fp64 oracle."""
import numpy as np
import pytest

from taper_inputs import (AttnShape, bf16_bits_from_f32, f32_from_bf16_bits, fill_values_numpy, structure_config3,
                          structure_custom)
from tests.gpu_util import assert_parity, bits_from_torch, run_gpu, run_oracle, torch_bf16

pytestmark = pytest.mark.gpu

QWEN = AttnShape(64, 8, 128, 16)
RAGGED = [(37, [0]), (50, [0, 7, 16, 21]), (16, [1]), (700, [0, 33, 64, 65, 129, 300]), (1, [0]), (2100, [0]),
          (0, [45]), (31, [31, 32, 33]), (64, [0, 0]), (129, [1] * 9)]
POOL_REQS = [(2100, [0]), (900, [0]), (1500, [5, 60, 0, 17, 130, 40, 3, 3, 250]), (640, [700, 1, 33]), (77, [0]),
             (3000, [0]), (16, [1]), (1200, [12] * 20)]
FINE = dict(target_workgroups=2048, min_share_tokens=1)  # many partials per sequence


def new_ctx(**kw):
    from paper_2605_06914_amd import Context

    return Context(64, 8, 128, device=0, **kw)


@pytest.mark.parametrize("reqs,kw", [(RAGGED, {}), (POOL_REQS, {}), (POOL_REQS, FINE),
                                     (POOL_REQS, dict(max_branches_per_item=24)),
                                     ([(333, [int(x) for x in range(40)]), (300, [0])], {})],
                         ids=["ragged", "pool", "pool_fine", "pool_wide_items", "width40"])
def test_fp32_partial_rows_meet_the_same_bar(reqs, kw):
    """partial_format = fp32: the other route between workgroups, same parity bar, same lse."""
    ctx = new_ctx(partial_format="f32")
    b = fill_values_numpy(structure_custom(QWEN, reqs, seed=501))
    ref, ref_lse = run_oracle(b)
    got, lse, bits = run_gpu(ctx, b, **kw)
    assert_parity(got, ref, f"fp32 partial rows {kw}")
    assert np.max(np.abs(lse - ref_lse)) <= 2e-3
    _, _, again = run_gpu(ctx, b, **kw)
    assert np.array_equal(bits, again)
    ctx.close()


@pytest.mark.parametrize("partial_format", ["f16_scaled", "f32"])
@pytest.mark.parametrize("log2_scale", [-60, 13, 20, 100])
def test_values_of_v_far_beyond_the_half_precision_range(partial_format, log2_scale):
    """V times 2^s (|V| up to 1e31 at s = 100, down to 1e-18 at s = -60; bf16 holds both): the result must be the
    unscaled result times 2^s whatever format the partial rows travel in -- no overflow to Inf, no flush to
    zero -- with the sequences cut so finely that nearly every output goes through partials."""
    ctx = new_ctx(partial_format=partial_format)
    b = fill_values_numpy(structure_custom(QWEN, POOL_REQS, seed=141))
    ref, _ = run_oracle(b)
    base, _, _ = run_gpu(ctx, b, **FINE)
    assert_parity(base, ref, "unscaled")
    st, sh = b.structure, b.structure.shape
    kv = b.kv.reshape(st.n_pool_pages, 2, sh.n_kv_heads, sh.page_size * sh.head_dim)
    v = f32_from_bf16_bits(kv[:, 1]) * np.float32(2.0 ** log2_scale)  # exact: a power of two
    kv[:, 1] = bf16_bits_from_f32(v)
    if log2_scale >= 13:
        assert np.abs(v).max() > (65504 if log2_scale > 13 else 1e4)
    got, _, _ = run_gpu(ctx, b, **FINE)
    assert np.isfinite(got).all()
    back = got / 2.0 ** log2_scale
    assert_parity(back, ref, f"V x 2^{log2_scale}, {partial_format}")
    assert np.max(np.abs(back - base)) <= 1e-3
    ctx.close()


def test_a_graph_captured_from_a_plan_survives_a_larger_plan():
    """Capture the launches of plan A, then build a plan B that needs a larger workspace (it gets one of its
    own) and run it, then replay A's graph: the bits of the eager run of A, every time."""
    import torch

    ctx = new_ctx()
    a = fill_values_numpy(structure_custom(QWEN, POOL_REQS, seed=131))
    sa = a.structure
    qa, kva = torch_bf16(a.q), torch_bf16(a.kv)
    plan_a = ctx.plan_build(sa.block_table, sa.branch_group, sa.prefix_len, sa.suffix_len, sa.n_pool_pages)
    ea = plan_a.export()
    eager = torch.full_like(qa, float("nan"))
    ctx.decode_step_attention(plan_a, qa, kva, eager)
    torch.cuda.synchronize()
    ref, _ = run_oracle(a)
    assert_parity(f32_from_bf16_bits(bits_from_torch(eager)).astype(np.float64), ref, "plan A eager")

    out = torch.full_like(qa, float("nan"))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            ctx.decode_step_attention(plan_a, qa, kva, out)
    torch.cuda.current_stream().wait_stream(side)

    b = fill_values_numpy(structure_config3())  # 22k partial rows against A's few thousand
    sb = b.structure
    qb, kvb = torch_bf16(b.q), torch_bf16(b.kv)
    plan_b = ctx.plan_build(sb.block_table, sb.branch_group, sb.prefix_len, sb.suffix_len, sb.n_pool_pages)
    eb = plan_b.export()
    assert eb["n_partial_rows"] > ea["workspace_rows"] and eb["workspace_id"] != ea["workspace_id"]
    assert plan_a.export()["workspace_id"] == ea["workspace_id"]
    out_b = torch.full_like(qb, float("nan"))
    for replay in range(3):
        out.fill_(float("nan"))
        ctx.decode_step_attention(plan_b, qb, kvb, out_b)  # B's launches between the replays of A
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), eager.view(torch.int16)), f"replay {replay}"
    ref_b, _ = run_oracle(b)
    assert_parity(f32_from_bf16_bits(bits_from_torch(out_b)).astype(np.float64), ref_b, "plan B")
    plan_a.free()
    plan_b.free()
    ctx.close()


def test_partial_rows_of_an_earlier_batch_do_not_leak():
    """Two different batches back to back on one context (the second finds the first one's partial rows and
    statistics in the workspace), against the second batch alone on a fresh context: same bits.  A merge
    that read a row before its writer had delivered it would pick up the other batch's numbers."""
    first = fill_values_numpy(structure_custom(QWEN, POOL_REQS, seed=601))
    second = fill_values_numpy(structure_custom(QWEN, [(1800, [9, 0, 40, 77, 5]), (2500, [0]), (640, [3, 700]), (90, [0]),
                                                       (1300, [1] * 11)], seed=602))
    used = new_ctx()
    for kw in ({}, FINE):
        _, _, _ = run_gpu(used, first, **kw)
        _, _, bits_after = run_gpu(used, second, **kw)
        fresh = new_ctx()
        got, _, bits_alone = run_gpu(fresh, second, **kw)
        fresh.close()
        assert np.array_equal(bits_after, bits_alone), f"{kw}"
        ref, _ = run_oracle(second)
        assert_parity(got, ref, f"second batch {kw}")
    used.close()


def test_reserve_then_no_growth():
    """taper_reserve sizes the workspace once; plans up to that size bind to it."""
    ctx = new_ctx()
    b = fill_values_numpy(structure_custom(QWEN, POOL_REQS, seed=131))
    st = b.structure
    ctx.reserve(max_seqs=256, max_partial_rows=200000)
    ids = set()
    for kw in ({}, FINE):
        plan = ctx.plan_build(st.block_table, st.branch_group, st.prefix_len, st.suffix_len, st.n_pool_pages, **kw)
        ids.add(plan.export()["workspace_id"])
        plan.free()
    assert ids == {1}
    ref, _ = run_oracle(b)
    got, _, _ = run_gpu(ctx, b)
    assert_parity(got, ref, "after reserve")
    ctx.close()


def test_two_batches_taking_turns_repeat_their_bits():
    """Two different batches, finely cut (thousands of partial rows each, the same workspace), launched in
    turns without a host synchronisation between the launches, 150 times each: every result must be the bits
    of the first.  The partial rows, statistics and counters of one launch are what the next one finds in the
    workspace; a merge that ran ahead of a writer, a counter that did not return to zero or a row picked up
    from the other batch would change bits sooner or later."""
    import torch

    ctx = new_ctx()
    batches = [fill_values_numpy(structure_custom(QWEN, POOL_REQS, seed=611)),
               fill_values_numpy(structure_custom(QWEN, [(1800, [9, 0, 40, 77, 5]), (2500, [0]), (640, [3, 700]), (90, [0]),
                                                         (1300, [1] * 11)], seed=612))]
    dev = []
    for b in batches:
        st = b.structure
        plan = ctx.plan_build(st.block_table, st.branch_group, st.prefix_len, st.suffix_len, st.n_pool_pages, **FINE)
        q, kv = torch_bf16(b.q), torch_bf16(b.kv)
        first = torch.full_like(q, float("nan"))
        ctx.decode_step_attention(plan, q, kv, first)
        torch.cuda.synchronize()
        ref, _ = run_oracle(b)
        assert_parity(f32_from_bf16_bits(bits_from_torch(first)).astype(np.float64), ref, "first launch")
        dev.append((plan, q, kv, first, [torch.empty_like(q) for _ in range(6)]))
    assert dev[0][0].export()["workspace_id"] == dev[1][0].export()["workspace_id"]
    for rnd in range(25):
        for k in range(6):  # 12 launches in a row on the stream, then compare
            for plan, q, kv, _, outs in dev:
                ctx.decode_step_attention(plan, q, kv, outs[k])
        torch.cuda.synchronize()
        for which, (_, _, _, first, outs) in enumerate(dev):
            for k in range(6):
                assert torch.equal(outs[k].view(torch.int16), first.view(torch.int16)), f"round {rnd}, launch {k}, batch {which}"
    for plan, *_ in dev:
        plan.free()
    ctx.close()
