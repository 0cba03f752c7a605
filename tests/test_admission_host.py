"""The library's predictor fit and per-step planner (C ABI, host only) against the
oracle in oracle/admission.py: coefficients to rounding, integer grants bit-exact."""
import numpy as np
import pytest

from oracle import admission as ora
from paper_2605_06914_amd import TaperError, Window, admit_step, predictor_eval, predictor_fit, predictor_mape
from paper_2605_06914_amd import TAPER_EINVAL, TAPER_ELEN


def grid_observations(rng, noise=0.02):
    batches = np.unique(np.round(np.geomspace(1, 512, 20)))
    ctxs = np.linspace(128, 8192, 25)
    n, c = np.meshgrid(batches, ctxs, indexing="ij")
    n, L = n.ravel(), (n * c).ravel()
    t = (0.31 + 0.0042 * n + 5.1e-7 * L) * (1 + rng.normal(0, noise, n.shape))
    return n, L, t


@pytest.mark.parametrize("noise", [0.0, 0.02, 0.3])
def test_fit_matches_oracle(noise):
    n, L, t = grid_observations(np.random.default_rng(3), noise)
    coef, mape = predictor_fit(n, L, t)
    ref = ora.predictor_fit(n, L, t)
    assert np.allclose(coef, ref, rtol=1e-9, atol=1e-12)
    assert mape == pytest.approx(ora.mape_pct(ref, n, L, t), rel=1e-9, abs=1e-9)
    assert predictor_mape(coef, n, L, t) == pytest.approx(mape, rel=1e-12)
    assert predictor_eval(coef, 100, 50000) == pytest.approx(ora.predictor_eval(ref, 100, 50000), rel=1e-12)


def probe_like_observations(seed):
    """16 steps (batch 1-64 x context 128-8192) whose small ones are launch-bound and noisy."""
    rng = np.random.default_rng(seed)
    n = np.repeat([1.0, 4.0, 16.0, 64.0], 4)
    L = n * np.tile([128.0, 1024.0, 4096.0, 8192.0], 4)
    t = 0.03 + 1.2e-6 * L + rng.normal(-2e-4, 3e-4) * n + rng.normal(0, 2e-3, 16)
    return n, L, t


@pytest.mark.parametrize("seed", range(12))
def test_monotone_fit_matches_oracle_and_is_usable_by_the_planner(seed):
    """A refresh never hands the planner a model it refuses: b, c >= 0, equal to the oracle's bounded least
    squares, and equal to the plain fit whenever that is monotone already."""
    n, L, t = probe_like_observations(seed)
    coef, mape = predictor_fit(n, L, t, monotone=True)
    ref = ora.predictor_fit_monotone(n, L, t)
    assert np.allclose(coef, ref, rtol=1e-6, atol=1e-11), (coef, ref)
    assert coef[1] >= 0 and coef[2] >= 0
    assert mape == pytest.approx(ora.mape_pct(coef, n, L, t), rel=1e-9)
    free, _ = predictor_fit(n, L, t)
    if free[1] >= 0 and free[2] >= 0:
        assert np.allclose(coef, free, rtol=1e-9, atol=1e-13)
    else:
        assert coef[1] == 0.0 or coef[2] == 0.0
        with pytest.raises(TaperError):  # the plain fit is what the planner refuses
            admit_step(free, [100, 100], [1e3, 1e3], [[50], []])
    granted, res = admit_step(coef, [100, 100], [1e3, 1e3], [[50], []])
    assert granted.tolist() == [1, 0] and np.isfinite(res["t_pred_ms"])


def test_some_probe_like_sets_do_need_the_constraint():
    assert any(predictor_fit(*probe_like_observations(s))[0][1] < 0 for s in range(12))


def test_window_refresh_is_monotone():
    w = Window(16)
    n, L, t = probe_like_observations(next(s for s in range(12) if predictor_fit(*probe_like_observations(s))[0][1] < 0))
    for x in zip(n, L, t):
        w.push(*x)
    free, _ = w.fit()
    coef, _ = w.fit(monotone=True)
    assert free[1] < 0 and coef[1] == 0.0 and coef[2] > 0
    assert np.allclose(coef, ora.predictor_fit_monotone(n, L, t), rtol=1e-6, atol=1e-11)
    w.close()


def test_fit_hand_example():
    coef, mape = predictor_fit([1, 1, 3, 3], [1, 3, 1, 3], [2, 4, 6, 12])
    assert np.allclose(coef, (-4, 3, 2), atol=1e-12) and mape == pytest.approx(25.0)


def test_fit_rejects_degenerate_observations():
    too_few = ([1, 2], [1, 2], [1, 2])
    same_batch = ([4, 4, 4, 4], [1, 2, 3, 5], [1, 2, 3, 4])              # batch size never varies
    proportional = ([1, 2, 3, 4], [10, 20, 30, 40], [1, 2, 3, 4])        # context proportional to batch
    not_finite = ([1, 2, 3, 4], [1, 5, 2, 8], [1, 2, float("nan"), 4])
    for args in (too_few, same_batch, proportional, not_finite):
        with pytest.raises(TaperError) as e:
            predictor_fit(*args)
        assert e.value.status == TAPER_EINVAL
    for args in (same_batch, proportional):  # the oracle agrees that these do not determine (a, b, c)
        with pytest.raises(ValueError):
            ora.predictor_fit(*args)


def test_window_keeps_the_most_recent_steps():
    rng = np.random.default_rng(9)
    obs = []
    w = Window(200)
    for i in range(520):
        n = int(rng.integers(1, 513))
        L = n * int(rng.integers(128, 8193))
        drift = 1.0 + i / 1000.0  # the machine slows down over time
        t = (0.3 + 0.004 * n + 5e-7 * L) * drift
        obs.append((n, L, t))
        w.push(n, L, t)
        if i in (2, 150, 199, 200, 519):
            assert len(w) == min(i + 1, 200)
            if i >= 150:
                coef, _ = w.fit()
                assert np.allclose(coef, ora.rolling_fit(obs, window=200), rtol=1e-8)
    w.close()


def random_case(rng, n_req, kind):
    base = rng.integers(1, 9000, n_req)
    slack = rng.uniform(1.0, 60.0, n_req)
    branches = [[int(b + rng.integers(0, 2049)) for _ in range(int(rng.integers(0, 18)))] if rng.random() < 0.5 else []
                for b in base]
    weight = rng.integers(1, 5, n_req).astype(float)
    table = None
    if kind == "table":
        table = [np.concatenate([[0.0], np.cumsum(rng.integers(0, 3, len(b)).astype(float))]) for b in branches]
    return base, slack, branches, weight, table


@pytest.mark.parametrize("kind", ["linear", "concave", "table"])
def test_planner_matches_oracle(kind):
    rng = np.random.default_rng({"linear": 1, "concave": 2, "table": 3}[kind])
    coef = (0.8, 0.011, 2.3e-6)
    for trial in range(200):
        n_req = int(rng.integers(1, 40))
        base, slack, branches, weight, table = random_case(rng, n_req, kind)
        rho = float(rng.uniform(0.05, 1.0))
        if trial % 7 == 0:
            slack = slack * 100  # ample slack: everything is admitted
        granted, res = admit_step(coef, base, slack, branches, rho=rho, utility=kind, weight=weight, utility_table=table)
        reqs = [ora.Request(int(base[r]), float(slack[r]), branches[r],
                            ora.utility_curve(kind, float(weight[r]), None if table is None else table[r]))
                for r in range(n_req)]
        ref = ora.taper_step(reqs, coef, rho)
        assert granted.tolist() == ref.granted, (kind, trial)
        assert (res["n_tokens"], res["l_context"], res["evaluations"]) == (ref.n_tokens, ref.l_context, ref.evaluations)
        assert res["admitted"] == sum(ref.granted)
        assert res["t0_ms"] == pytest.approx(ref.t0, rel=1e-12) and res["budget_ms"] == pytest.approx(ref.budget, rel=1e-12)
        assert res["t_pred_ms"] == pytest.approx(ref.t_pred, rel=1e-12)
        assert res["t_pred_ms"] <= res["budget_ms"] + 1e-12


def test_planner_worked_example():
    coef = (1.0, 0.1, 0.001)
    g, res = admit_step(coef, [1000, 2000, 500], [50, 20, 100], [[], [2000, 2100, 2200], [500, 600]], rho=0.5)
    assert g.tolist() == [0, 2, 2] and res["evaluations"] == 7
    assert res["budget_ms"] == pytest.approx(12.4) and res["t_pred_ms"] == pytest.approx(10.4)
    g, res = admit_step(coef, [1000, 2000, 500], [8, 20, 100], [[], [2000, 2100, 2200], [500, 600]], rho=0.5)
    assert g.tolist() == [0, 0, 2] and res["evaluations"] == 3


def test_planner_rejects_bad_arguments():
    ok = dict(coef=(1.0, 0.1, 0.001), base_context=[10, 20], slack_ms=[5.0, 6.0], branch_context=[[10], []])
    for over, code in ((dict(rho=0.0), TAPER_EINVAL), (dict(rho=1.5), TAPER_EINVAL), (dict(coef=(1.0, -0.1, 0.001)), TAPER_EINVAL),
                       (dict(base_context=[10, -1]), TAPER_ELEN), (dict(branch_context=[[-5], []]), TAPER_ELEN),
                       (dict(slack_ms=[float("nan"), 1.0]), TAPER_EINVAL)):
        with pytest.raises(TaperError) as e:
            admit_step(**{**ok, **over})
        assert e.value.status == code
