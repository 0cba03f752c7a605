"""GPU parity: the HIP library (through its C ABI) against the fp64 oracle, element
by element, on the same seeded inputs.  Bar: max-abs 2e-2, mean-abs 2e-3 for the
floating-point outputs (bf16 inputs, fp32 accumulation); integers bit-exact."""
import numpy as np
import pytest

import oracle
from taper_inputs import (AttnShape, Batch, bf16_bits_from_f32, compact_rows, f32_from_bf16_bits, fill_values_numpy,
                          structure_config1, structure_config2, structure_config3, structure_custom)
from tests.gpu_util import assert_parity, bits_from_torch, run_gpu, run_oracle, torch_bf16
from tests.layout_ref import PoolView

pytestmark = pytest.mark.gpu

QWEN = AttnShape(64, 8, 128, 16)
TINY = AttnShape(4, 1, 64, 16)


@pytest.fixture(scope="module")
def ctx_qwen():
    from paper_2605_06914_amd import Context

    c = Context(64, 8, 128, device=0)
    yield c
    c.close()


@pytest.fixture(scope="module")
def ctx_tiny():
    from paper_2605_06914_amd import Context

    c = Context(4, 1, 64, device=0)
    yield c
    c.close()


def test_library_is_loaded_from_tree():
    from paper_2605_06914_amd import LIB_PATH, load_library

    load_library()
    assert any(LIB_PATH in line for line in open("/proc/self/maps"))


@pytest.mark.parametrize("share", [True, False])
def test_config1_tiny(ctx_tiny, share):
    b = fill_values_numpy(structure_config1())
    ref, ref_lse = run_oracle(b)
    got, lse, _ = run_gpu(ctx_tiny, b, share_prefix=share)
    assert_parity(got, ref, f"config1 share={share}")
    assert np.max(np.abs(lse - ref_lse)) <= 2e-3


RAGGED = [(37, [0]), (50, [0, 7, 16, 21]), (16, [1]), (700, [0, 33, 64, 65, 129, 300]), (1, [0]), (2100, [0]),
          (0, [45]), (31, [31, 32, 33]), (64, [0, 0]), (129, [1] * 9)]


@pytest.mark.parametrize("share,target", [(True, 0), (False, 0), (True, 8), (True, 4096), (True, -4096)])
def test_ragged_qwen_shape(ctx_qwen, share, target):
    """Several tiles, partial pages, prefixes ending mid-page, empty branches, a
    suffix-only sequence, one-token context; also under very coarse and very fine
    workgroup shares."""
    b = fill_values_numpy(structure_custom(QWEN, RAGGED, seed=101))
    ref, ref_lse = run_oracle(b)
    kw = dict(target_workgroups=target) if target >= 0 else dict(target_workgroups=-target, min_share_tokens=1)
    got, lse, _ = run_gpu(ctx_qwen, b, share_prefix=share, **kw)
    assert_parity(got, ref, f"ragged share={share} target={target}")
    assert np.max(np.abs(lse - ref_lse)) <= 2e-3


@pytest.mark.parametrize("width", [2, 3, 16, 17, 24, 25, 40, 65, 130])
def test_wide_requests(ctx_qwen, width):
    """Branch widths around the limits of one workgroup's row tiles (16 rows per
    tile, 12 tiles per workgroup, wider requests cut into sub-groups)."""
    rng = np.random.default_rng(width)
    reqs = [(300, [0]), (333, [int(x) for x in rng.integers(0, 40, size=width)])]
    b = fill_values_numpy(structure_custom(QWEN, reqs, seed=200 + width))
    ref, _ = run_oracle(b)
    got, _, _ = run_gpu(ctx_qwen, b)
    assert_parity(got, ref, f"width={width}")


@pytest.mark.parametrize("width", [5, 48, 50])
def test_wide_requests_tiny_shape(ctx_tiny, width):
    rng = np.random.default_rng(width)
    reqs = [(90, [int(x) for x in rng.integers(0, 40, size=width)]), (77, [0])]
    b = fill_values_numpy(structure_custom(TINY, reqs, seed=300 + width))
    ref, _ = run_oracle(b)
    got, _, _ = run_gpu(ctx_tiny, b)
    assert_parity(got, ref, f"tiny width={width}")


def poison(b: Batch, val=1e30, bits=None):
    """+-val (or the two given bf16 bit patterns) in every slot no sequence may read."""
    st, sh = b.structure, b.structure.shape
    P = sh.page_size
    valid = np.zeros((st.n_pool_pages, P), bool)
    for s in range(st.n_seqs):
        npre, nsuf = int(st.prefix_len[s]), int(st.suffix_len[s])
        npp = -(-npre // P)
        for t in range(npre):
            valid[st.block_table[s, t // P], t % P] = True
        for j in range(nsuf):
            valid[st.block_table[s, npp + j // P], j % P] = True
    pv = PoolView(sh.n_kv_heads, sh.head_dim, P)
    flat = b.kv.reshape(-1)
    d = np.arange(sh.head_dim)
    pos = bf16_bits_from_f32(np.array([val], np.float32))[0]
    neg = bf16_bits_from_f32(np.array([-val], np.float32))[0]
    if bits is not None:
        pos, neg = np.uint16(bits[0]), np.uint16(bits[1])
    pages, toks = np.nonzero(~valid)
    for page, tok in zip(pages, toks):
        for hk in range(sh.n_kv_heads):
            flat[pv.k_off(page, hk, tok, d)] = np.where(d % 2 == 0, pos, neg)
            flat[pv.v_off(page, hk, tok, d)] = np.where(d % 2 == 0, neg, pos)


def test_garbage_in_invalid_slots_changes_nothing(ctx_qwen):
    reqs = [(37, [0]), (50, [0, 7, 16, 21]), (16, [1]), (133, [3, 70])]
    b = fill_values_numpy(structure_custom(QWEN, reqs, seed=102))
    _, _, bits0 = run_gpu(ctx_qwen, b)
    poison(b)
    got, _, bits1 = run_gpu(ctx_qwen, b)
    ref, _ = run_oracle(b)
    assert_parity(got, ref, "poisoned")
    assert np.array_equal(bits0, bits1)


@pytest.mark.parametrize("bits", [(0x7FC0, 0xFFC0), (0x7F80, 0xFF80), (0x7FC0, 0x7F80)], ids=["nan", "inf", "nan_inf"])
@pytest.mark.parametrize("share", [1, 0])
def test_nan_and_inf_in_invalid_slots_change_nothing(ctx_qwen, bits, share):
    """Unwritten slots of a half-filled page may hold any bits, NaN and Inf included (pages come
    from an allocator, not zeroed): K there is masked after the scores, V there must not meet
    its zero weight as 0 * NaN.  Both the shared-prefix and the per-sequence kernels' tails."""
    reqs = [(37, [0]), (50, [0, 7, 16, 21]), (16, [1]), (133, [3, 70]), (1, [0]), (15, [17, 1]), (17, [15, 33])]
    b = fill_values_numpy(structure_custom(QWEN, reqs, seed=105))
    _, _, bits0 = run_gpu(ctx_qwen, b, share_prefix=share)
    poison(b, bits=bits)
    got, _, bits1 = run_gpu(ctx_qwen, b, share_prefix=share)
    assert np.isfinite(got).all()
    assert np.array_equal(bits0, bits1)


def test_run_to_run_bit_identical(ctx_qwen):
    b = fill_values_numpy(structure_custom(QWEN, RAGGED, seed=103))
    import torch

    q, kv = torch_bf16(b.q), torch_bf16(b.kv)
    runs = [run_gpu(ctx_qwen, b, q, kv)[2] for _ in range(3)]
    assert np.array_equal(runs[0], runs[1]) and np.array_equal(runs[0], runs[2])


POOL_REQS = [(2100, [0]), (900, [0]), (1500, [5, 60, 0, 17, 130, 40, 3, 3, 250]), (640, [700, 1, 33]), (77, [0]),
             (3000, [0]), (16, [1]), (1200, [12] * 20)]


@pytest.mark.parametrize("kw", [dict(pool_pct=-1), dict(pool_pct=90, pool_item_tokens=64), dict(pool_pct=50),
                                dict(pool_pct=25, target_workgroups=64),
                                dict(shared_cost_pct=300, shared_item_cost=5000, private_item_cost=1),
                                dict(max_branches_per_item=3), dict(max_branches_per_item=24),
                                dict(max_branches_per_item=8, pool_pct=75, pool_item_tokens=200)])
def test_plan_options_do_not_change_the_result(ctx_qwen, kw):
    """The unowned pool of private items (claimed at run time by workgroups that
    finish early), the cost weights and the branch cap only move work between
    workgroups; every setting must meet the same parity bar."""
    b = fill_values_numpy(structure_custom(QWEN, POOL_REQS, seed=107))
    ref, ref_lse = run_oracle(b)
    got, lse, _ = run_gpu(ctx_qwen, b, **kw)
    assert_parity(got, ref, f"options {kw}")
    assert np.max(np.abs(lse - ref_lse)) <= 2e-3


@pytest.mark.parametrize("width", [17, 20, 24])
def test_wide_requests_in_one_pass(ctx_qwen, width):
    """Requests of 9 to 12 row tiles served by one item per prefix chunk (the kernel variant that loads
    straight into LDS, four 32-token buffers): prefix lengths around every block and page boundary,
    so one to many blocks, odd page counts and ragged tails; narrower requests ride in the same launch."""
    rng = np.random.default_rng(400 + width)
    reqs = [(pl, [int(x) for x in rng.integers(0, 40, size=width)]) for pl in (1, 15, 16, 17, 31, 32, 33, 63, 64, 65, 95, 96, 97, 129, 1000)]
    reqs += [(77, [0]), (300, [5, 0, 9]), (2500, [int(x) for x in rng.integers(0, 90, size=width)]), (500, [1] * 9)]
    b = fill_values_numpy(structure_custom(QWEN, reqs, seed=400 + width))
    ref, ref_lse = run_oracle(b)
    got, lse, bits0 = run_gpu(ctx_qwen, b, max_branches_per_item=24)
    assert_parity(got, ref, f"wide {width}")
    assert np.max(np.abs(lse - ref_lse)) <= 2e-3
    poison(b, bits=(0x7FC0, 0xFF80))
    _, _, bits1 = run_gpu(ctx_qwen, b, max_branches_per_item=24)
    assert np.array_equal(bits0, bits1)
    _, _, bits2 = run_gpu(ctx_qwen, b, max_branches_per_item=24, target_workgroups=8)
    got2 = f32_from_bf16_bits(bits2).astype(np.float64)
    assert_parity(got2, ref, f"wide {width}, 8 workgroups")


def test_same_plan_replayed(ctx_qwen):
    """The arrival counters and the pool's claim counter reset themselves inside the
    kernel: replaying one plan must give the same bits every time."""
    import torch

    b = fill_values_numpy(structure_custom(QWEN, POOL_REQS, seed=108))
    st = b.structure
    q, kv = torch_bf16(b.q), torch_bf16(b.kv)
    plan = ctx_qwen.plan_build(st.block_table, st.branch_group, st.prefix_len, st.suffix_len, st.n_pool_pages,
                               pool_pct=60, pool_item_tokens=128)
    assert plan.export()["n_pool_items"] > 0
    bits = []
    for _ in range(6):
        out = torch.full_like(q, float("nan"))
        ctx_qwen.decode_step_attention(plan, q, kv, out)
        torch.cuda.synchronize()
        bits.append(bits_from_torch(out))
    plan.free()
    ref, _ = run_oracle(b)
    assert_parity(f32_from_bf16_bits(bits[0]).astype(np.float64), ref, "replayed plan")
    for x in bits[1:]:
        assert np.array_equal(bits[0], x)


def test_many_partials_per_sequence(ctx_qwen):
    """Very fine shares: a sequence's partials number in the hundreds, far more than one merge round holds
    and more than the item-start prefetch of merge entries covers (the rest is fetched during the merge)."""
    reqs = [(9000, [0]), (6000, [3, 0, 70, 1, 200, 16, 5, 9, 130, 2, 31, 64, 8, 4, 77, 12]), (40, [0])]
    b = fill_values_numpy(structure_custom(QWEN, reqs, seed=109))
    st = b.structure
    plan = ctx_qwen.plan_build(st.block_table, st.branch_group, st.prefix_len, st.suffix_len, st.n_pool_pages,
                               target_workgroups=8192, pool_pct=-1, min_share_tokens=1)
    e = plan.export()
    per_seq = np.diff(e["merge_start"])
    plan.free()
    assert per_seq[0] > 128 and per_seq[1:17].sum() > 128 and per_seq[1] > 8
    ref, ref_lse = run_oracle(b)
    got, lse, _ = run_gpu(ctx_qwen, b, target_workgroups=8192, pool_pct=-1, min_share_tokens=1)
    assert_parity(got, ref, f"{int(per_seq.max())} partials per sequence")
    assert np.max(np.abs(lse - ref_lse)) <= 2e-3


@pytest.mark.parametrize("hq,hkv,d", [(16, 1, 128), (8, 8, 64), (6, 2, 128), (32, 8, 64), (64, 4, 128)])
def test_other_head_shapes(hq, hkv, d):
    """Group sizes 1, 3, 4, 16 (the largest supported) and both head dims, on a ragged batch with wide requests."""
    from paper_2605_06914_amd import Context

    sh = AttnShape(hq, hkv, d, 16)
    reqs = RAGGED + [(333, [int(x) for x in np.random.default_rng(hq).integers(0, 60, size=21)])]
    b = fill_values_numpy(structure_custom(sh, reqs, seed=110 + hq))
    ctx = Context(hq, hkv, d, device=0)
    try:
        ref, ref_lse = run_oracle(b)
        for kw in ({}, dict(target_workgroups=2048)):
            got, lse, _ = run_gpu(ctx, b, **kw)
            assert_parity(got, ref, f"shape Hq{hq} Hkv{hkv} D{d} {kw}")
            assert np.max(np.abs(lse - ref_lse)) <= 2e-3
    finally:
        ctx.close()


def test_head_dim_64_with_three_tiles_per_wave():
    """head_dim 64 serves 9 to 12 row tiles per item only when asked to (the variant stages through registers
    and runs one workgroup per compute unit): 40 branches x 4 query heads per KV head = 10 tiles."""
    from paper_2605_06914_amd import Context

    sh = AttnShape(32, 8, 64, 16)
    rng = np.random.default_rng(64)
    reqs = [(pl, [int(x) for x in rng.integers(0, 50, size=40)]) for pl in (1, 63, 64, 65, 200, 1500)] + [(90, [0]), (40, [3, 0, 5])]
    b = fill_values_numpy(structure_custom(sh, reqs, seed=164))
    ctx = Context(32, 8, 64, device=0)
    try:
        ref, ref_lse = run_oracle(b)
        st = b.structure
        plan = ctx.plan_build(st.block_table, st.branch_group, st.prefix_len, st.suffix_len, st.n_pool_pages, max_branches_per_item=48)
        e = plan.export()
        plan.free()
        assert int(e["items"][:, e["item_fields"].index("n_branch")].max()) == 40
        got, lse, _ = run_gpu(ctx, b, max_branches_per_item=48)
        assert_parity(got, ref, "D64, 10 row tiles")
        assert np.max(np.abs(lse - ref_lse)) <= 2e-3
        got, _, _ = run_gpu(ctx, b)  # default: cut into sub-groups of at most 8 tiles
        assert_parity(got, ref, "D64, default cap")
    finally:
        ctx.close()


@pytest.mark.parametrize("kw", [{}, dict(solo_item_tokens=-1), dict(solo_item_tokens=64), dict(target_workgroups=64)])
def test_many_short_sequences(ctx_qwen, kw):
    """Batches of short serial requests: each sequence is one item whose result the kernel writes directly
    (no partial rows), and runs of them are worked on by single waves, four side by side."""
    rng = np.random.default_rng(12)
    reqs = [(int(n), [0]) for n in rng.integers(1, 300, size=700)] + [(2000, [0]), (5, [3, 0])] + \
           [(0, [int(n)]) for n in rng.integers(1, 200, size=40)]
    b = fill_values_numpy(structure_custom(QWEN, reqs, seed=111))
    st = b.structure
    plan = ctx_qwen.plan_build(st.block_table, st.branch_group, st.prefix_len, st.suffix_len, st.n_pool_pages, **kw)
    e = plan.export()
    plan.free()
    kinds = np.bincount(e["items"][:, e["item_fields"].index("kind")], minlength=4)
    assert kinds[2] + kinds[3] >= 700
    if kw.get("solo_item_tokens", 0) == -1:
        assert kinds[3] == 0
    elif kw.get("solo_item_tokens", 0) == 0:
        assert kinds[3] > 100
    ref, ref_lse = run_oracle(b)
    got, lse, _ = run_gpu(ctx_qwen, b, **kw)
    assert_parity(got, ref, f"short sequences {kw} kinds {kinds.tolist()}")
    assert np.max(np.abs(lse - ref_lse)) <= 2e-3


@pytest.mark.parametrize("gain", [0.02, 8.0, 40.0])
def test_flat_and_peaked_softmax(ctx_qwen, gain):
    """Scores scaled down (all weights nearly equal) and far up (one token takes almost all the weight, scores
    of several thousand): the running maximum keeps every exponent in range."""
    b = fill_values_numpy(structure_custom(QWEN, RAGGED, seed=112))
    q = f32_from_bf16_bits(b.q) * np.float32(gain)
    b = Batch(b.structure, bf16_bits_from_f32(q), b.kv)
    ref, ref_lse = run_oracle(b)
    got, lse, _ = run_gpu(ctx_qwen, b)
    assert_parity(got, ref, f"q scaled by {gain}")
    assert np.max(np.abs(lse - ref_lse) / np.maximum(1.0, np.abs(ref_lse))) <= 2e-3


def test_sibling_independence(ctx_qwen):
    """Lemma 1: which siblings share the step must not change a branch's output
    (beyond summation order; the prefix partial is computed per row, so it is in
    fact bit-identical as long as the chunking of the prefix is the same)."""
    reqs = [(500, [0]), (900, [5, 60, 0, 17, 130, 40])]
    b = fill_values_numpy(structure_custom(QWEN, reqs, seed=104))
    full, _, _ = run_gpu(ctx_qwen, b)
    ref, _ = run_oracle(b)
    assert_parity(full, ref, "all siblings")
    worst = 0.0
    for keep in ([0, 3], [0, 1, 6], [0, 6, 4, 2]):
        rows = np.array(sorted(keep))
        sub, pages = compact_rows(b.structure, rows)
        bs = Batch(sub, b.q[rows], b.kv[pages])
        got, _, _ = run_gpu(ctx_qwen, bs)
        assert_parity(got, ref[rows], f"siblings {keep}")
        worst = max(worst, float(np.max(np.abs(got - full[rows]))))
    print(f"[lemma1] max |out(subset) - out(all)| = {worst:.3e}")
    assert worst <= 4e-3


def test_dominant_key_names_the_physical_slot(ctx_qwen):
    """End-to-end index check through the floating-point path: one key aligned
    with q takes all the weight and V rows are one-hot codes of (page, token)."""
    sh = AttnShape(64, 8, 128, 16)
    st = structure_custom(sh, [(24, [0]), (20, [3, 20])], seed=6, n_pool_pages=7)
    b = fill_values_numpy(st)
    pv = PoolView(8, 128, 16)
    flat = b.kv.reshape(-1)
    d = np.arange(128)
    one = bf16_bits_from_f32(np.array([1.0], np.float32))[0]
    for page in range(7):
        for tok in range(16):
            for hk in range(8):
                flat[pv.v_off(page, hk, tok, d)] = np.where(d == page * 16 + tok, one, 0).astype(np.uint16)
    rng = np.random.default_rng(0)
    for s in range(st.n_seqs):
        npre, nsuf = int(st.prefix_len[s]), int(st.suffix_len[s])
        for t_star in [int(rng.integers(0, npre))] + ([npre + int(rng.integers(0, nsuf))] if nsuf else []):
            if t_star < npre:
                page, tok = int(st.block_table[s, t_star // 16]), t_star % 16
            else:
                j = t_star - npre
                page, tok = int(st.block_table[s, -(-npre // 16) + j // 16]), j % 16
            h = int(rng.integers(0, 64))
            qv = f32_from_bf16_bits(b.q[s, h]).astype(np.float64)
            saved = flat[pv.k_off(page, h // 8, tok, d)].copy()
            flat[pv.k_off(page, h // 8, tok, d)] = bf16_bits_from_f32((200.0 * qv / np.linalg.norm(qv)).astype(np.float32))
            got, _, _ = run_gpu(ctx_qwen, b)
            flat[pv.k_off(page, h // 8, tok, d)] = saved
            assert int(np.argmax(got[s, h])) == page * 16 + tok
            assert got[s, h, page * 16 + tok] == 1.0
            assert np.count_nonzero(got[s, h]) == 1


@pytest.mark.parametrize("maker", [structure_config1, lambda: structure_custom(QWEN, RAGGED, seed=101)])
def test_integer_outputs_bit_exact(maker):
    import torch

    from paper_2605_06914_amd import Context

    st = maker()
    sh = st.shape
    ints = oracle.resolve(sh.page_size, st.block_table, st.branch_group, st.prefix_len, st.suffix_len)
    ctx = Context(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, device=0)
    plan = ctx.plan_build(st.block_table, st.branch_group, st.prefix_len, st.suffix_len, st.n_pool_pages)
    e = plan.export()
    assert e["n_groups"] == ints.n_groups
    for key in ("ctx_len", "n_prefix_pages", "n_suffix_pages", "group_start"):
        assert np.array_equal(e[key], getattr(ints, key)), key
    stride = ints.slots.shape[1]
    dev = torch.full((st.n_seqs, stride), -7, dtype=torch.int64, device="cuda:0")
    plan.resolve_slots(dev, stride)
    torch.cuda.synchronize()
    assert np.array_equal(dev.cpu().numpy(), ints.slots)
    assert np.array_equal(plan.resolve_slots_host(stride), ints.slots)
    plan.free()
    ctx.close()


def test_simple_entry_point(ctx_qwen):
    import torch

    b = fill_values_numpy(structure_custom(QWEN, RAGGED[:4], seed=105))
    st = b.structure
    q, kv = torch_bf16(b.q), torch_bf16(b.kv)
    out = torch.zeros_like(q)
    ctx_qwen.decode_step_attention_simple(q, kv, st.n_pool_pages, st.block_table, st.branch_group, st.prefix_len,
                                          st.suffix_len, out)
    got = f32_from_bf16_bits(bits_from_torch(out)).astype(np.float64)
    ref, _ = run_oracle(b)
    assert_parity(got, ref, "simple entry")


def test_step_latency_probe_runs(ctx_qwen):
    import torch

    b = fill_values_numpy(structure_custom(QWEN, RAGGED, seed=106))
    st = b.structure
    q, kv = torch_bf16(b.q), torch_bf16(b.kv)
    outs = [torch.zeros_like(q) for _ in range(3)]
    plan = ctx_qwen.plan_build(st.block_table, st.branch_group, st.prefix_len, st.suffix_len, st.n_pool_pages)
    res = ctx_qwen.step_latency_probe(plan, [q] * 3, [kv] * 3, outs, warmup=2, iters=5)
    assert res.n_tokens == st.n_seqs and res.n_layers == 3
    assert res.l_context == st.logical_tokens
    assert res.kv_bytes_unique == st.kv_bytes_unique and res.kv_bytes_logical == st.kv_bytes_logical
    assert 0 < res.us_min <= res.us_median
    ref, _ = run_oracle(b)
    for o in outs:
        assert_parity(f32_from_bf16_bits(bits_from_torch(o)).astype(np.float64), ref, "probe layer")
    kt = ctx_qwen.kernel_times(plan, q, kv, outs[0], warmup=1, iters=3)
    assert kt["decode_us"] >= kt["decode_us_min"] > 0
    kt = ctx_qwen.kernel_times_layers(plan, [q] * 3, [kv] * 3, outs, warmup=1, iters=4)
    assert kt["decode_us"] >= kt["decode_us_min"] > 0
    plan.free()


def test_config2_full_size(ctx_qwen):
    """IRP-Off batch at full size, default launch configuration, every output."""
    b = fill_values_numpy(structure_config2())
    ref, _ = run_oracle(b)
    got, _, _ = run_gpu(ctx_qwen, b, want_lse=False)
    assert_parity(got, ref, "config2 full")


def test_config3_full_size(ctx_qwen):
    """Mixed batch at full size, default launch configuration, every output of all 68 sequences."""
    b = fill_values_numpy(structure_config3())
    ref, ref_lse = run_oracle(b)
    got, lse, _ = run_gpu(ctx_qwen, b)
    assert_parity(got, ref, "config3 full")
    assert np.max(np.abs(lse - ref_lse)) <= 2e-3


def sample_rows(st, n_serial=8):
    sizes = np.bincount(st.branch_group)
    serial = [s for s in range(st.n_seqs) if sizes[st.branch_group[s]] == 1]
    rows = serial[:: max(1, len(serial) // n_serial)][:n_serial]
    for g in np.flatnonzero(sizes > 1):
        m = np.flatnonzero(st.branch_group == g)
        rows += [int(m[0]), int(m[-1])]
    return sorted(set(rows))


def test_config4_long_context_sampled(ctx_qwen):
    """Long-context batch at full size: 8 requests with a 32768-token prefix and 16 branches plus 32 serial
    requests, pages scattered in a ~30 GB pool (64-bit addressing, 458k pages).  The oracle checks 8 serial
    sequences and every request's first and last branch, all heads; all outputs must be finite."""
    import torch

    from taper_inputs import structure_config4
    from tests.gpu_util import device_random_batch, host_subbatch, run_gpu_device

    st = structure_config4()
    assert st.n_pool_pages * st.shape.page_elems * 2 > 29e9
    q, kv = device_random_batch(st)
    out = run_gpu_device(ctx_qwen, st, q, kv)
    assert bool(torch.isfinite(out.float()).all())
    rows, sub = host_subbatch(st, q, kv, sample_rows(st))
    del kv
    torch.cuda.empty_cache()
    ref, _ = run_oracle(sub)
    got = f32_from_bf16_bits(bits_from_torch(out[torch.from_numpy(rows).to(out.device)])).astype(np.float64)
    assert_parity(got, ref, "config4 sampled")


@pytest.mark.parametrize("k", [0, 2, 4, 8, 16])
def test_config5_sweep_point_sampled(ctx_qwen, k):
    """One layer of the admission sweep at full size (96 serial + 32 parallel requests, width 1+k)."""
    import torch

    from taper_inputs import structure_config5
    from tests.gpu_util import device_random_batch, host_subbatch, run_gpu_device

    st = structure_config5(k)
    assert st.n_seqs == 96 + 32 * (1 + k)
    q, kv = device_random_batch(st)
    out = run_gpu_device(ctx_qwen, st, q, kv)
    assert bool(torch.isfinite(out.float()).all())
    rows, sub = host_subbatch(st, q, kv, sample_rows(st, n_serial=6)[:40])
    del kv
    torch.cuda.empty_cache()
    ref, _ = run_oracle(sub)
    got = f32_from_bf16_bits(bits_from_torch(out[torch.from_numpy(rows).to(out.device)])).astype(np.float64)
    assert_parity(got, ref, f"config5 k={k} sampled")


def test_config5_k16_every_output_two_ways(ctx_qwen):
    """k = 16 at full size through both routes for 17-branch requests: one item of 9 row tiles per prefix
    chunk (loads straight into LDS) and two sub-groups of 9 + 8 branches (register staging).  Every
    output of the step is compared, not a sample; the one-pass route is replayed and must repeat its bits
    (its barriers and waits are hand-placed: a race would show as a changing bit)."""
    import torch

    from taper_inputs import structure_config5
    from tests.gpu_util import device_random_batch

    st = structure_config5(16)
    q, kv = device_random_batch(st)
    outs = []
    for cap in (24, 24, 24, 24, 16):
        plan = ctx_qwen.plan_build(st.block_table, st.branch_group, st.prefix_len, st.suffix_len, st.n_pool_pages,
                                   max_branches_per_item=cap)
        e = plan.export()
        F = {n: i for i, n in enumerate(e["item_fields"])}
        assert int(e["items"][:, F["n_branch"]].max()) == (17 if cap == 24 else 9)
        out = torch.full_like(q, float("nan"))
        ctx_qwen.decode_step_attention(plan, q, kv, out)
        torch.cuda.synchronize()
        plan.free()
        outs.append(out)
    for o in outs[1:4]:
        assert torch.equal(outs[0].view(torch.int16), o.view(torch.int16))
    a, b = outs[0].float(), outs[4].float()
    assert bool(torch.isfinite(a).all()) and bool(torch.isfinite(b).all())
    assert float((a - b).abs().max()) <= 2e-2 and float((a - b).abs().mean()) <= 2e-3


def test_layer_launches_replay_from_a_captured_graph(ctx_qwen):
    """The attention call is one kernel launch on the caller's stream (no memset, no allocation, no host wait), so a
    stack of layers can be captured once per plan and replayed.  Several replays, with eager work and
    synchronisations between them, must each reproduce the eager bits (the arrival and pool counters put
    themselves back to zero inside the kernel)."""
    import torch

    b = fill_values_numpy(structure_custom(QWEN, POOL_REQS, seed=131))
    st = b.structure
    n_layers = 6
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(5)
    kvs = [torch_bf16(b.kv)] + [torch.randn(b.kv.size, generator=gen, device="cuda:0").to(torch.bfloat16) for _ in range(n_layers - 1)]
    qs = [torch_bf16(b.q)] + [torch.randn(b.q.shape, generator=gen, device="cuda:0").to(torch.bfloat16) for _ in range(n_layers - 1)]
    plan = ctx_qwen.plan_build(st.block_table, st.branch_group, st.prefix_len, st.suffix_len, st.n_pool_pages)
    eager = [torch.full_like(qs[0], float("nan")) for _ in range(n_layers)]
    for l in range(n_layers):
        ctx_qwen.decode_step_attention(plan, qs[l], kvs[l], eager[l])
    torch.cuda.synchronize()
    ref, _ = run_oracle(b)
    assert_parity(f32_from_bf16_bits(bits_from_torch(eager[0])).astype(np.float64), ref, "eager layer 0")

    outs = [torch.full_like(qs[0], float("nan")) for _ in range(n_layers)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            for l in range(n_layers):
                ctx_qwen.decode_step_attention(plan, qs[l], kvs[l], outs[l])
    torch.cuda.current_stream().wait_stream(side)
    for replay in range(4):
        for o in outs:
            o.fill_(float("nan"))
        scratch = torch.full_like(qs[0], float("nan"))
        ctx_qwen.decode_step_attention(plan, qs[replay % n_layers], kvs[replay % n_layers], scratch)  # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for l in range(n_layers):
            assert torch.equal(outs[l].view(torch.int16), eager[l].view(torch.int16)), f"replay {replay}, layer {l}"
    plan.free()


@pytest.mark.parametrize("log2_scale", [9, 13])
def test_large_values_of_v_pass_through_the_partials(ctx_qwen, log2_scale):
    """V scaled by 2^9 and 2^13 (|V| up to about 3e4) must give the unscaled result times the same power of two
    (partial rows between workgroups travel normalised and scaled row by row; larger factors and the fp32
    format are covered in test_gpu_robustness.py)."""
    b = fill_values_numpy(structure_custom(QWEN, POOL_REQS, seed=141))
    base, _, _ = run_gpu(ctx_qwen, b, target_workgroups=2048, min_share_tokens=1)
    st, sh = b.structure, b.structure.shape
    pv = PoolView(sh.n_kv_heads, sh.head_dim, sh.page_size)
    kv = b.kv.reshape(st.n_pool_pages, 2, sh.n_kv_heads, sh.page_size * sh.head_dim)
    v = f32_from_bf16_bits(kv[:, 1]) * np.float32(2.0 ** log2_scale)  # exact: a power of two
    kv[:, 1] = bf16_bits_from_f32(v)
    assert np.abs(v).max() < 65504
    got, _, _ = run_gpu(ctx_qwen, b, target_workgroups=2048, min_share_tokens=1)
    assert np.isfinite(got).all()
    assert np.max(np.abs(got / 2.0 ** log2_scale - base)) <= 1e-3


def test_five_thousand_sequences(ctx_qwen):
    """A step far wider than the paper's batches (5000 sequences: short serial requests and two-branch requests
    with tiny prefixes): counters, merge lists and partial rows are indexed per sequence and must scale."""
    rng = np.random.default_rng(151)
    reqs = []
    for _ in range(4000):
        reqs.append((int(rng.integers(1, 48)), [0]))
    for _ in range(500):
        reqs.append((int(rng.integers(1, 80)), [int(rng.integers(0, 20)), int(rng.integers(0, 20))]))
    b = fill_values_numpy(structure_custom(QWEN, reqs, seed=151))
    assert b.structure.n_seqs == 5000
    ref, ref_lse = run_oracle(b)
    for kw in ({}, dict(share_prefix=0, target_workgroups=4096)):
        got, lse, _ = run_gpu(ctx_qwen, b, **kw)
        assert_parity(got, ref, f"5000 sequences {kw}")
        assert np.max(np.abs(lse - ref_lse)) <= 2e-3
