"""GPU test of the entry point that allocates nothing (taper_decode_step_attention_static):
its result must equal, bit for bit, that of taper_decode_step_attention_simple on the same
inputs -- both build the same plan and the merge order is fixed by the plan -- and meet the
oracle bar; on two calls in a row, the second with a smaller input, so that what the first
call left in the library's scratch array must not matter."""
import numpy as np
import pytest

from taper_inputs import AttnShape, fill_values_numpy, structure_config1, structure_config3, structure_custom
from tests.gpu_util import assert_parity, bits_from_torch, run_oracle, torch_bf16

pytestmark = pytest.mark.gpu

QWEN = AttnShape(64, 8, 128, 16)
BIG = [(700, [0, 33, 64, 65, 129, 300]), (2100, [0]), (37, [0]), (50, [0, 7, 16, 21]), (0, [45]), (1500, [5] * 9),
       (3000, [0]), (129, [1] * 20)]
SMALL = [(50, [0, 7]), (333, [0]), (16, [1])]


def both_ways(ctx, b):
    import torch

    st = b.structure
    q, kv = torch_bf16(b.q), torch_bf16(b.kv)
    args = (q, kv, st.n_pool_pages, st.block_table, st.branch_group, st.prefix_len, st.suffix_len)
    out_static = torch.full_like(q, float("nan"))
    ctx.decode_step_attention_static(*args, out_static)
    torch.cuda.synchronize()
    out_simple = torch.full_like(q, float("nan"))
    ctx.decode_step_attention_simple(*args, out_simple)
    torch.cuda.synchronize()
    return bits_from_torch(out_static), bits_from_torch(out_simple)


@pytest.mark.parametrize("partial_format", ["f16_scaled", "f32"])
def test_static_entry_matches_the_allocating_one_on_two_calls_in_a_row(partial_format):
    from paper_2605_06914_amd import Context
    from taper_inputs import f32_from_bf16_bits

    ctx = Context(64, 8, 128, device=0, partial_format=partial_format)
    for name, reqs, seed in (("first, larger", BIG, 401), ("second, smaller", SMALL, 402)):
        b = fill_values_numpy(structure_custom(QWEN, reqs, seed=seed))
        print(f"[no-alloc] {partial_format} {name}: S={b.structure.n_seqs}", flush=True)
        got, want = both_ways(ctx, b)
        assert np.array_equal(got, want), f"{name}: static entry differs from the allocating one"
        ref, _ = run_oracle(b)
        assert_parity(f32_from_bf16_bits(got).astype(np.float64), ref, f"static entry, {name}")
    ctx.close()


def test_static_entry_on_the_mixed_batch_and_the_tiny_shape():
    from paper_2605_06914_amd import Context
    from taper_inputs import f32_from_bf16_bits

    ctx = Context(64, 8, 128, device=0)
    b = fill_values_numpy(structure_config3())
    print(f"[no-alloc] mixed batch: S={b.structure.n_seqs}", flush=True)
    got, want = both_ways(ctx, b)
    assert np.array_equal(got, want)
    ctx.close()
    tiny = Context(4, 1, 64, device=0)  # another context on the same GPU shares the array
    b = fill_values_numpy(structure_config1())
    print("[no-alloc] tiny shape after it", flush=True)
    got, want = both_ways(tiny, b)
    assert np.array_equal(got, want)
    ref, _ = run_oracle(b)
    assert_parity(f32_from_bf16_bits(got).astype(np.float64), ref, "static entry, tiny shape")
    tiny.close()


def test_static_entry_rejects_a_step_beyond_the_array():
    import torch

    from paper_2605_06914_amd import Context, TaperError, TAPER_EINVAL

    # 6000 sequences of one page each, every one cut off from sharing: the plan image is small but a block table
    # of 6000 x 9000 entries is not (216 MB): the call must refuse before touching the device
    ctx = Context(64, 8, 128, device=0)
    S, width = 6000, 9000
    bt = np.zeros((S, width), np.int32)
    q = torch.zeros((S, 64, 128), dtype=torch.bfloat16, device="cuda:0")
    kv = torch.zeros(16 * QWEN.page_elems, dtype=torch.bfloat16, device="cuda:0")
    out = torch.zeros_like(q)
    with pytest.raises(TaperError) as e:
        ctx.decode_step_attention_static(q, kv, 16, bt, np.arange(S, dtype=np.int32), np.full(S, 5, np.int32),
                                         np.zeros(S, np.int32), out)
    assert e.value.status == TAPER_EINVAL and "static scratch" in str(e.value)
    ctx.close()
