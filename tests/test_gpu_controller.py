"""GPU side of the controller rows: the predictor is fitted from probe timings of real
steps (library fit against the oracle's on the same measurements), and a step composed
by the planner runs through the kernels and meets the attention parity bar."""
import numpy as np
import pytest

from oracle import admission as ora
from taper_inputs import Batch, build_structure, compact_rows, fill_values_numpy, structure_config5, subset_rows
from taper_inputs.generators import QWEN
from tests.gpu_util import assert_parity, run_gpu, run_oracle, torch_bf16

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx_qwen():
    from paper_2605_06914_amd import Context

    c = Context(64, 8, 128, device=0)
    yield c
    c.close()


def test_predictor_fitted_from_the_probe(ctx_qwen):
    import torch

    from paper_2605_06914_amd import predictor_fit, predictor_mape

    rng = np.random.Generator(np.random.PCG64(77))
    n_pool_pages = 40000  # 2.6 GB
    kv = torch.empty(n_pool_pages * QWEN.page_elems, device="cuda:0", dtype=torch.bfloat16).normal_()
    q = torch.randn((64, 64, 128), device="cuda:0").to(torch.bfloat16)
    out = torch.zeros_like(q)
    obs = []
    for b in (1, 4, 16, 64):
        for c in (128, 1024, 4096, 8192):
            st = build_structure(QWEN, [(c, [0])] * b, rng, n_pool_pages=n_pool_pages)
            plan = ctx_qwen.plan_build(st.block_table, st.branch_group, st.prefix_len, st.suffix_len, n_pool_pages)
            r = ctx_qwen.step_latency_probe(plan, [q[:b]] * 2, [kv] * 2, [out[:b]] * 2, warmup=2, iters=5)
            plan.free()
            assert r.n_tokens == b and r.l_context == b * c and r.us_median > 0
            obs.append((b, b * c, r.us_median / 1e3))
    n, L, t = (np.array(x, np.float64) for x in zip(*obs))
    coef, mape = predictor_fit(n, L, t)
    ref = ora.predictor_fit(n, L, t)
    assert np.allclose(coef, ref, rtol=1e-8, atol=1e-12)
    assert mape == pytest.approx(ora.mape_pct(ref, n, L, t), rel=1e-8)
    assert predictor_mape(coef, n, L, t) == pytest.approx(mape, rel=1e-12)
    print(f"[predictor] a={coef[0]:.4f} ms b={coef[1]:.3e} c={coef[2]:.3e} MAPE {mape:.1f}%")
    assert coef[2] > 0  # more context costs more time
    # what a refresh hands the planner: the fit under b, c >= 0 (16 noisy, partly launch-bound steps can give the
    # plain fit a negative slope on the batch size, which the planner refuses)
    mono, mono_mape = predictor_fit(n, L, t, monotone=True)
    assert mono[1] >= 0 and mono[2] > 0
    assert np.allclose(mono, ora.predictor_fit_monotone(n, L, t), rtol=1e-6, atol=1e-11)
    if coef[1] >= 0:
        assert np.allclose(mono, coef, rtol=1e-9, atol=1e-13)
    from paper_2605_06914_amd import admit_step
    granted, res = admit_step(mono, [1024, 1024], [1e3, 1e3], [[100, 100], []])
    assert granted.tolist() == [2, 0]
    print(f"[predictor, monotone] a={mono[0]:.4f} ms b={mono[1]:.3e} c={mono[2]:.3e} MAPE {mono_mape:.1f}%")
    # the largest step streams 2.1 GB per layer: its time is set by HBM, not by launch overheads
    assert t[-1] > 10 * t[0]


def test_step_composed_by_the_planner_meets_parity(ctx_qwen):
    from paper_2605_06914_amd import admit_step

    full = structure_config5(16, n_serial=10, n_parallel=4)
    first = np.flatnonzero(np.r_[True, full.branch_group[1:] != full.branch_group[:-1]])
    sizes = np.bincount(full.branch_group)
    base = (full.prefix_len + full.suffix_len)[first].astype(np.int64)
    ready = [[int(full.suffix_len[s]) for s in range(first[g] + 1, first[g] + sizes[g])] for g in range(full.n_groups)]
    coef = (0.04, 3.6e-4, 2.4e-6)  # ms; the shape of a fit on unique tokens
    t0 = coef[0] + coef[1] * full.n_groups + coef[2] * base.sum()
    slack = np.full(full.n_groups, 1e9)
    slack[2] = 1.35 * t0
    granted, res = admit_step(coef, base, slack, ready, rho=1.0, utility="concave")
    reqs = [ora.Request(int(base[g]), float(slack[g]), ready[g], ora.utility_curve("concave")) for g in range(full.n_groups)]
    assert granted.tolist() == ora.taper_step(reqs, coef, 1.0).granted
    assert 0 < res["admitted"] < sum(len(r) for r in ready) and np.all(granted[:10] == 0)
    rows = np.concatenate([first[g] + np.arange(1 + granted[g]) for g in range(full.n_groups)])
    st = subset_rows(full, rows)
    assert st.n_seqs == full.n_groups + res["admitted"] == res["n_tokens"]
    sub, pages = compact_rows(st, np.arange(st.n_seqs))  # compact pool so that the host oracle can hold it
    b = fill_values_numpy(sub)
    ref, _ = run_oracle(b)
    got, _, _ = run_gpu(ctx_qwen, b)
    assert_parity(got, ref, f"planner-composed step, {res['admitted']} opportunistic branches")
