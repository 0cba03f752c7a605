"""CPU-only tests of the workspace bookkeeping (host-only contexts keep the same records as
device contexts, without the device memory): a plan stays bound to the workspace it was built
with whatever is built later, so that launches in flight and captured graphs keep valid
addresses; and of the binding's checks of the tensors it is handed."""
import pytest

from paper_2605_06914_amd import Context, TaperError, TAPER_EINVAL
from taper_inputs import AttnShape, structure_config2, structure_config3, structure_custom

QWEN = AttnShape(64, 8, 128, 16)


def build(ctx, st, **kw):
    return ctx.plan_build(st.block_table, st.branch_group, st.prefix_len, st.suffix_len, st.n_pool_pages, **kw)


def test_a_larger_plan_gets_a_workspace_of_its_own_and_leaves_the_old_one_alone():
    ctx = Context(64, 8, 128, device=-1)
    small = build(ctx, structure_custom(QWEN, [(700, [0, 33, 64]), (2100, [0])], seed=1))
    a = small.export()
    assert a["workspace_id"] == 1 and a["workspace_rows"] >= a["n_partial_rows"]
    big = build(ctx, structure_config3())
    b = big.export()
    assert b["n_partial_rows"] > a["workspace_rows"], "the second plan must not fit the first workspace"
    assert b["workspace_id"] == 2 and b["workspace_rows"] >= b["n_partial_rows"]
    again = small.export()  # the first plan still sits where it sat
    assert again["workspace_id"] == 1 and again["workspace_rows"] == a["workspace_rows"]
    # a plan that fits the current workspace shares it, also a small one
    third = build(ctx, structure_custom(QWEN, [(50, [0, 7])], seed=2))
    assert third.export()["workspace_id"] == 2
    for p in (small, big, third):
        p.free()
    # steady state: the same batch again and again never moves
    ids = set()
    for _ in range(5):
        p = build(ctx, structure_config3())
        ids.add(p.export()["workspace_id"])
        p.free()
    assert ids == {2}
    ctx.close()


def test_reserve_sizes_the_workspace_ahead_of_time():
    ctx = Context(64, 8, 128, device=-1)
    probe = build(ctx, structure_config3())
    rows = probe.export()["n_partial_rows"]
    probe.free()
    ctx2 = Context(64, 8, 128, device=-1)
    ctx2.reserve(max_seqs=128, max_partial_rows=rows)
    p = build(ctx2, structure_config3())
    e = p.export()
    assert e["workspace_id"] == 1 and e["workspace_rows"] >= rows
    q = build(ctx2, structure_config2())
    assert q.export()["workspace_id"] == 1
    p.free()
    q.free()
    ctx2.reserve(max_seqs=1, max_partial_rows=1)  # smaller than what is there: nothing happens
    r = build(ctx2, structure_config3())
    assert r.export()["workspace_id"] == 1
    r.free()
    with pytest.raises(TaperError) as err:
        ctx2.reserve(-1, 5)
    assert err.value.status == TAPER_EINVAL
    ctx.close()
    ctx2.close()


def test_unknown_partial_format_is_rejected():
    with pytest.raises(TaperError) as err:
        Context(64, 8, 128, device=-1, partial_format=7)
    assert err.value.status == TAPER_EINVAL
    for fmt in ("f16_scaled", "f32"):
        Context(64, 8, 128, device=-1, partial_format=fmt).close()


class FakeTensor:
    """What the binding looks at of a torch tensor (no GPU here)."""

    class Dev:
        def __init__(self, type_, index):
            self.type, self.index = type_, index

        def __repr__(self):
            return f"{self.type}:{self.index}"

    def __init__(self, numel, dtype="torch.bfloat16", contiguous=True, device=("cuda", 0)):
        self._n, self.dtype, self._c, self.device = numel, dtype, contiguous, self.Dev(*device)

    def numel(self):
        return self._n

    def is_contiguous(self):
        return self._c

    def data_ptr(self):
        return 4096  # never dereferenced: the context is host-only, the library would answer TAPER_EHIP


@pytest.mark.parametrize("what,bad", [
    ("q", dict(numel=68 * 64 * 128 - 1)), ("q", dict(dtype="torch.float16")), ("q", dict(contiguous=False)),
    ("q", dict(device=("cpu", None))), ("q", dict(device=("cuda", 1))),
    ("kv", dict(numel=100)), ("kv", dict(dtype="torch.float32")),
    ("out", dict(numel=5)), ("out", dict(contiguous=False)),
    ("lse", dict(dtype="torch.bfloat16")), ("lse", dict(numel=68 * 64 - 1))])
def test_binding_refuses_tensors_the_kernel_would_overrun(what, bad):
    """dtype, contiguity, device and size are checked on the host, before any launch."""
    st = structure_config3()
    ctx = Context(64, 8, 128, device=-1)
    plan = build(ctx, st)
    ctx.cfg.device = 0  # pretend it is a device context: the tensor checks come before the library call
    sizes = dict(q=st.n_seqs * 64 * 128, out=st.n_seqs * 64 * 128, kv=st.n_pool_pages * 2 * 8 * 16 * 128,
                 lse=st.n_seqs * 64)
    dtypes = dict(q="torch.bfloat16", out="torch.bfloat16", kv="torch.bfloat16", lse="torch.float32")
    args = {}
    for name in sizes:
        kw = dict(numel=sizes[name], dtype=dtypes[name])
        if name == what:
            kw.update(bad)
        args[name] = FakeTensor(**kw)
    with pytest.raises(TaperError) as err:
        ctx.decode_step_attention(plan, args["q"], args["kv"], args["out"], args["lse"], stream=0)
    assert err.value.status == TAPER_EINVAL and {"kv": "kv_pages"}.get(what, what) in str(err.value)
    ctx.cfg.device = -1
    plan.free()
    ctx.close()
