"""Helpers for the GPU parity tests: move a seeded batch to the device, run the
library through its C ABI, bring the result back as float64."""
import numpy as np

import oracle
from taper_inputs import Batch, f32_from_bf16_bits

MAX_ABS, MEAN_ABS = 2e-2, 2e-3  # parity bar for bf16 inputs / fp32 accumulation


def torch_bf16(bits: np.ndarray, device="cuda:0"):
    import torch

    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device)
    return t.view(torch.bfloat16)


def bits_from_torch(t) -> np.ndarray:
    import torch

    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def run_gpu(ctx, b: Batch, q_dev=None, kv_dev=None, want_lse=True, **plan_kw):
    """Returns (out float64 [S,Hq,D], lse float64 or None, out bits uint16)."""
    import torch

    st, sh = b.structure, b.structure.shape
    q_dev = torch_bf16(b.q) if q_dev is None else q_dev
    kv_dev = torch_bf16(b.kv) if kv_dev is None else kv_dev
    out = torch.full((st.n_seqs, sh.n_q_heads, sh.head_dim), float("nan"), dtype=torch.bfloat16, device=q_dev.device)
    lse = torch.full((st.n_seqs, sh.n_q_heads), float("nan"), dtype=torch.float32, device=q_dev.device) if want_lse else None
    plan = ctx.plan_build(st.block_table, st.branch_group, st.prefix_len, st.suffix_len, st.n_pool_pages, **plan_kw)
    ctx.decode_step_attention(plan, q_dev, kv_dev, out, lse)
    torch.cuda.synchronize()
    plan.free()
    bits = bits_from_torch(out)
    return (f32_from_bf16_bits(bits).astype(np.float64), lse.double().cpu().numpy() if want_lse else None, bits)


def run_oracle(b: Batch, n_threads=0):
    st, sh = b.structure, b.structure.shape
    out, lse, _, _ = oracle.attention(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.page_size, sh.scale, b.q, b.kv,
                                      st.block_table, st.prefix_len, st.suffix_len, n_threads=n_threads)
    return out, lse


def assert_parity(got, ref, what=""):
    assert np.all(np.isfinite(got)), f"{what}: non-finite output"
    err = np.abs(got - ref)
    rms = float(np.sqrt(np.mean(ref ** 2)))
    mx, mean = float(err.max()), float(err.mean())
    print(f"[parity] {what}: max_abs={mx:.3e} mean_abs={mean:.3e} rms(ref)={rms:.3e} max_abs/rms={mx / rms:.3e}", flush=True)
    if mx > MAX_ABS and err.ndim == 3:  # name the rows that are off: which sequences, which heads
        per_row = err.max(axis=2)
        bad = np.argwhere(per_row > MAX_ABS)
        print(f"[parity] {what}: {len(bad)} (sequence, head) rows above the bar; first: "
              + ", ".join(f"(s={s}, h={h}: {per_row[s, h]:.3e})" for s, h in bad[:: max(1, len(bad) // 24)]), flush=True)
    assert mx <= MAX_ABS, f"{what}: max-abs {mx} > {MAX_ABS}"
    assert mean <= MEAN_ABS, f"{what}: mean-abs {mean} > {MEAN_ABS}"
    # the absolute bar is loose for long contexts (outputs shrink like 1/sqrt(n)); bf16 rounding of the
    # output alone is 2^-9 relative per element, so hold each sequence's error to a few percent of that
    # sequence's own output scale too
    ax = tuple(range(1, ref.ndim))
    rms_s = np.sqrt(np.mean(ref ** 2, axis=ax))
    rel = err.max(axis=ax) / (rms_s + 1e-12)
    worst = int(np.argmax(rel))
    assert rel[worst] <= 0.05, f"{what}: sequence {worst}: max-abs {err[worst].max()} is more than 5% of its rms {rms_s[worst]}"
    return mx, mean


def device_random_batch(st, seed=None, device="cuda:0"):
    """q and the whole pool drawn on the device (N(0,1) rounded to bf16); for pools too big for numpy."""
    import torch

    sh = st.shape
    gen = torch.Generator(device=device)
    gen.manual_seed((st.seed + 1000) if seed is None else seed)
    q = torch.randn((st.n_seqs, sh.n_q_heads, sh.head_dim), generator=gen, device=device).to(torch.bfloat16)
    n = st.n_pool_pages * sh.page_elems
    kv = torch.empty(n, device=device, dtype=torch.bfloat16)
    chunk = 1 << 28
    for o in range(0, n, chunk):
        m = min(chunk, n - o)
        kv[o : o + m] = torch.randn(m, generator=gen, device=device).to(torch.bfloat16)
    return q, kv


def host_subbatch(st, q_dev, kv_dev, rows):
    """The sequences `rows` with just the pages they reference, copied to the host."""
    import torch

    from taper_inputs import compact_rows

    rows = np.asarray(sorted(rows))
    sub, pages = compact_rows(st, rows)
    sh = st.shape
    pg = torch.from_numpy(pages).to(kv_dev.device)
    kv = bits_from_torch(kv_dev.view(st.n_pool_pages, sh.page_elems)[pg])
    q = bits_from_torch(q_dev[torch.from_numpy(rows).to(q_dev.device)])
    return rows, Batch(sub, q, kv)


def run_gpu_device(ctx, st, q_dev, kv_dev, **plan_kw):
    import torch

    out = torch.full_like(q_dev, float("nan"))
    plan = ctx.plan_build(st.block_table, st.branch_group, st.prefix_len, st.suffix_len, st.n_pool_pages, **plan_kw)
    ctx.decode_step_attention(plan, q_dev, kv_dev, out)
    torch.cuda.synchronize()
    plan.free()
    return out
