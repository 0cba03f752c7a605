"""GPU parity for the steps around the parallel phase: reduce-phase attention (contexts
made of several private segments), KV append (bit-exact), and a short decode loop that
alternates the two."""
import numpy as np
import pytest

import oracle
from taper_inputs import (AttnShape, bf16_bits_from_f32, f32_from_bf16_bits, fill_values_numpy, reduce_structure,
                          structure_custom)
from tests.gpu_util import assert_parity, bits_from_torch, torch_bf16

pytestmark = pytest.mark.gpu
QWEN = AttnShape(64, 8, 128, 16)
TINY = AttnShape(4, 1, 64, 16)


@pytest.fixture(scope="module")
def ctx_qwen():
    from paper_2605_06914_amd import Context

    c = Context(64, 8, 128, device=0)
    yield c
    c.close()


def parallel_batch(shape, seed, spare=200):
    reqs = [(37, [0]), (1500, [0, 7, 160, 21, 700]), (700, [0, 33, 64, 65, 129, 300, 2, 2]), (16, [1]), (2100, [0]),
            (333, list(range(0, 400, 21)))]
    st = structure_custom(shape, reqs, seed=seed)
    return fill_values_numpy(structure_custom(shape, reqs, seed=seed, n_pool_pages=st.n_pool_pages + spare))


def run_segments_gpu(ctx, seg, q_bits, kv_dev, **opts):
    import torch

    q = torch_bf16(q_bits)
    out = torch.full_like(q, float("nan"))
    lse = torch.full((seg.n_seqs, seg.shape.n_q_heads), float("nan"), dtype=torch.float32, device=q.device)
    plan = ctx.plan_build_segments(seg.block_table, seg.branch_group, seg.prefix_len, seg.seg_start, seg.seg_len,
                                   seg.n_pool_pages, **opts)
    ctx.decode_step_attention(plan, q, kv_dev, out, lse)
    torch.cuda.synchronize()
    return plan, f32_from_bf16_bits(bits_from_torch(out)).astype(np.float64), lse.double().cpu().numpy()


@pytest.mark.parametrize("keep,opts", [((), {}), ((1, 5), {}), ((2,), dict(target_workgroups=16)),
                                       ((1, 2, 5), dict(pool_pct=80, pool_item_tokens=64))])
def test_reduce_phase_attention(ctx_qwen, keep, opts):
    """Requests leaving their parallel phase (one reduce sequence over prefix + all branches + reduce tokens)
    next to requests still inside it (branches sharing a prefix) and serial ones."""
    import torch

    b = parallel_batch(QWEN, seed=31)
    seg = reduce_structure(b.structure, z_len=[0, 9, 130, 1, 17, 64], seed=32, keep_parallel=keep)
    rng = np.random.Generator(np.random.PCG64(33))
    q = bf16_bits_from_f32(rng.standard_normal((seg.n_seqs, 64, 128), dtype=np.float32))
    kv_dev = torch_bf16(b.kv)
    plan, got, lse = run_segments_gpu(ctx_qwen, seg, q, kv_dev, **opts)
    ref, ref_lse = oracle.attention_segments(64, 8, 128, 16, QWEN.scale, q, b.kv, seg.block_table, seg.prefix_len,
                                             seg.seg_start, seg.seg_len)
    assert_parity(got, ref, f"reduce phase keep={keep} {opts}")
    assert np.max(np.abs(lse - ref_lse)) <= 2e-3
    # integers: the device resolves every position to the slot the oracle names
    ctx_len, _, slots = oracle.resolve_segments(16, seg.block_table, seg.prefix_len, seg.seg_start, seg.seg_len)
    dev = torch.full(slots.shape, -7, dtype=torch.int64, device="cuda:0")
    plan.resolve_slots(dev, slots.shape[1])
    torch.cuda.synchronize()
    assert np.array_equal(dev.cpu().numpy(), slots)
    plan.free()


def test_reduce_phase_ignores_non_finite_bits_in_unwritten_slots(ctx_qwen):
    """A reduce sequence crosses the half-filled last page of every branch it absorbs: NaN / Inf
    bits in those pages' unwritten slots (and in pages nobody lists) must leave the result as it is."""
    from tests.layout_ref import PoolView

    b = parallel_batch(QWEN, seed=41)
    seg = reduce_structure(b.structure, z_len=[0, 9, 130, 1, 17, 64], seed=42, keep_parallel=(1, 5))
    rng = np.random.Generator(np.random.PCG64(43))
    q = bf16_bits_from_f32(rng.standard_normal((seg.n_seqs, 64, 128), dtype=np.float32))
    plan, got0, _ = run_segments_gpu(ctx_qwen, seg, q, torch_bf16(b.kv))
    plan.free()
    ctx_len, _, slots = oracle.resolve_segments(16, seg.block_table, seg.prefix_len, seg.seg_start, seg.seg_len)
    valid = np.zeros(seg.n_pool_pages * 16, bool)
    valid[slots[slots >= 0]] = True
    assert 0 < valid.sum() < valid.size
    pv = PoolView(8, 128, 16)
    kv = b.kv.copy()
    flat = kv.reshape(-1)
    d = np.arange(128)
    for slot in np.nonzero(~valid)[0]:
        page, tok = divmod(int(slot), 16)
        for hk in range(8):
            flat[pv.k_off(page, hk, tok, d)] = np.where(d % 3 == 0, 0x7FC0, np.where(d % 3 == 1, 0x7F80, 0xFF80)).astype(np.uint16)
            flat[pv.v_off(page, hk, tok, d)] = np.where(d % 3 == 0, 0xFF80, np.where(d % 3 == 1, 0x7FC0, 0x7F80)).astype(np.uint16)
    plan, got1, _ = run_segments_gpu(ctx_qwen, seg, q, torch_bf16(kv))
    plan.free()
    assert np.isfinite(got1).all()
    assert np.array_equal(got0, got1)


def test_kv_append_is_bit_exact(ctx_qwen):
    import torch

    from paper_2605_06914_amd import append_slots

    b = parallel_batch(QWEN, seed=41)
    st = b.structure
    S = st.n_seqs
    seg_start = np.arange(S + 1, dtype=np.int32)
    bt = np.concatenate([st.block_table, np.full((S, 1), -1, np.int32)], axis=1)
    used = set(int(x) for x in bt.ravel() if x >= 0)
    fresh = [p for p in range(st.n_pool_pages) if p not in used]
    for s in range(S):  # enter a page for every token that opens one
        if st.suffix_len[s] % 16 == 0:
            bt[s, -(-int(st.prefix_len[s]) // 16) + int(st.suffix_len[s]) // 16] = fresh.pop()
    slots, opens = append_slots(bt, st.prefix_len, seg_start, st.suffix_len, 16, st.n_pool_pages)
    assert len(set(slots.tolist())) == S and opens.sum() == np.sum(st.suffix_len % 16 == 0) > 0
    rng = np.random.Generator(np.random.PCG64(42))
    k_new = bf16_bits_from_f32(rng.standard_normal((S, 8, 128), dtype=np.float32))
    v_new = bf16_bits_from_f32(rng.standard_normal((S, 8, 128), dtype=np.float32))
    kv_dev = torch_bf16(b.kv)
    ctx_qwen.kv_append(torch_bf16(k_new), torch_bf16(v_new), torch.from_numpy(slots).to("cuda:0"), kv_dev, S)
    torch.cuda.synchronize()
    want = b.kv.copy()
    oracle.kv_append(8, 128, 16, k_new, v_new, slots, want)
    assert np.array_equal(bits_from_torch(kv_dev), want)
    assert np.count_nonzero(want != b.kv) > 0.99 * S * 2 * 8 * 128


def test_decode_loop_append_then_attend(ctx_qwen):
    """Four decode steps: every sequence's new K/V rows are appended (opening pages where needed), then the
    step's attention runs over the grown contexts.  Pool bytes stay identical to the oracle's; outputs meet
    the parity bar at every step."""
    import torch

    from paper_2605_06914_amd import append_slots, branch_blocks

    b = parallel_batch(QWEN, seed=51)
    par = b.structure
    seg = reduce_structure(par, z_len=[15, 16, 0, 31, 2, 48], seed=52, keep_parallel=(1, 5))
    S = seg.n_seqs
    bt = np.concatenate([seg.block_table, np.full((S, 2), -1, np.int32)], axis=1)
    used = set(int(x) for x in bt.ravel() if x >= 0)
    fresh = [p for p in range(seg.n_pool_pages) if p not in used]
    seg_len = seg.seg_len.copy()
    last = seg.seg_start[1:] - 1
    kv_host = b.kv.copy()
    kv_dev = torch_bf16(kv_host)
    rng = np.random.Generator(np.random.PCG64(53))
    pages_opened = 0
    for step in range(4):
        # host accounting: a sequence whose last segment fills its pages gets a page before the append
        for s in range(S):
            lens = seg_len[seg.seg_start[s]:seg.seg_start[s + 1]]
            if lens[-1] % 16 == 0:
                entry = -(-int(seg.prefix_len[s]) // 16) + sum(-(-int(n) // 16) for n in lens[:-1]) + int(lens[-1]) // 16
                bt[s, entry] = fresh.pop()
                pages_opened += 1
                assert branch_blocks(int(lens[-1]) + 1) == branch_blocks(int(lens[-1])) + 1
        slots, _ = append_slots(bt, seg.prefix_len, seg.seg_start, seg_len, 16, seg.n_pool_pages)
        k_new = bf16_bits_from_f32(rng.standard_normal((S, 8, 128), dtype=np.float32))
        v_new = bf16_bits_from_f32(rng.standard_normal((S, 8, 128), dtype=np.float32))
        ctx_qwen.kv_append(torch_bf16(k_new), torch_bf16(v_new), torch.from_numpy(slots).to("cuda:0"), kv_dev, S)
        oracle.kv_append(8, 128, 16, k_new, v_new, slots, kv_host)
        seg_len[last] += 1
        q = bf16_bits_from_f32(rng.standard_normal((S, 64, 128), dtype=np.float32))
        qd = torch_bf16(q)
        out = torch.full_like(qd, float("nan"))
        plan = ctx_qwen.plan_build_segments(bt, seg.branch_group, seg.prefix_len, seg.seg_start, seg_len, seg.n_pool_pages)
        ctx_qwen.decode_step_attention(plan, qd, kv_dev, out)
        torch.cuda.synchronize()
        plan.free()
        assert np.array_equal(bits_from_torch(kv_dev), kv_host), f"pool differs after step {step}"
        ref, _ = oracle.attention_segments(64, 8, 128, 16, QWEN.scale, q, kv_host, bt, seg.prefix_len, seg.seg_start, seg_len)
        assert_parity(f32_from_bf16_bits(bits_from_torch(out)).astype(np.float64), ref, f"decode loop step {step}")
    assert pages_opened >= 3


@pytest.mark.parametrize("seed", range(12))
def test_random_batches_and_options(ctx_qwen, seed):
    """Random mixes of serial requests, parallel phases (1-20 branches, empty suffixes included) and reduce
    sequences, under random plan options: same parity bar everywhere."""
    import torch

    rng = np.random.default_rng(1000 + seed)
    reqs = []
    for _ in range(int(rng.integers(3, 30))):
        kind = rng.integers(0, 4)
        if kind == 0:      # short serial
            reqs.append((int(rng.integers(1, 400)), [0]))
        elif kind == 1:    # long serial, context given as private tokens
            reqs.append((0, [int(rng.integers(500, 5000))]))
        else:              # parallel phase
            width = int(rng.choice([2, 3, 4, 7, 8, 9, 16, 17, 20]))
            reqs.append((int(rng.integers(1, 3000)), [int(x) for x in rng.integers(0, 300, size=width) * rng.integers(0, 2, size=width)]))
    st = structure_custom(QWEN, reqs, seed=2000 + seed)
    st = structure_custom(QWEN, reqs, seed=2000 + seed, n_pool_pages=st.n_pool_pages + 64)
    b = fill_values_numpy(st)
    n_groups = int(st.branch_group[-1]) + 1
    keep = [g for g in range(n_groups) if rng.random() < 0.6]
    seg = reduce_structure(st, z_len=[int(x) for x in rng.integers(0, 60, size=n_groups)], seed=seed, keep_parallel=keep)
    opts = {}
    if rng.random() < 0.5:
        opts["target_workgroups"] = int(rng.choice([8, 64, 256, 1024, 4096]))
    if rng.random() < 0.5:
        opts["pool_pct"] = int(rng.choice([-1, 10, 50, 90]))
    if rng.random() < 0.4:
        opts["min_share_tokens"] = int(rng.choice([1, 64, 1000]))
    if rng.random() < 0.3:
        opts["solo_item_tokens"] = int(rng.choice([-1, 32, 4096]))
    if rng.random() < 0.3:
        opts["max_branches_per_item"] = int(rng.choice([2, 5, 24]))
    if rng.random() < 0.2:
        opts["share_prefix"] = 0
    q = bf16_bits_from_f32(rng.standard_normal((seg.n_seqs, 64, 128), dtype=np.float32))
    kv_dev = torch_bf16(b.kv)
    plan, got, lse = run_segments_gpu(ctx_qwen, seg, q, kv_dev, **opts)
    plan.free()
    ref, ref_lse = oracle.attention_segments(64, 8, 128, 16, QWEN.scale, q, b.kv, seg.block_table, seg.prefix_len,
                                             seg.seg_start, seg.seg_len)
    assert_parity(got, ref, f"random batch {seed}: {seg.n_seqs} sequences, options {opts}")
    assert np.max(np.abs(lse - ref_lse)) <= 2e-3
