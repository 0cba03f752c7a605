"""Pins of the controller-side oracle (oracle/admission.py): the latency predictor of
App. C and the slack-budgeted greedy planner of §3.3-§3.4, against things that do not
come from the oracle itself: a hand-worked example (tests/golden/), closed forms,
defining properties, brute force over all grant vectors on tiny inputs.  The same
pins are run against planted mistakes to show that they can fail."""
import importlib.util
import itertools
import math
import os

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "admission.py")
G = os.path.join(ROOT, "tests", "golden")


def load_module(source=None, name="admission_under_test"):
    spec = importlib.util.spec_from_loader(name, loader=None)
    m = importlib.util.module_from_spec(spec)
    m.__dict__["__name__"] = name
    import sys
    sys.modules[name] = m  # dataclasses look the module up by name
    exec(compile(source if source is not None else open(SRC).read(), SRC, "exec"), m.__dict__)
    return m


def golden():
    d = {}
    for line in open(os.path.join(G, "admission_worked_example.txt")):
        f = line.split("#")[0].split()
        if f:
            d[f[0]] = [float(x) for x in f[1:]]
    return d


def example_requests(m, slack0=50.0):
    lin = m.utility_curve("linear", 1.0)
    return [m.Request(1000, slack0, [], lin), m.Request(2000, 20.0, [2000, 2100, 2200], lin),
            m.Request(500, 100.0, [500, 600], lin)]


COEF = (1.0, 0.1, 0.001)


# ---------------------------------------------------------------- predictor pins
def pin_ols_by_hand(m):
    g = golden()
    n, L, t = [1, 1, 3, 3], [1, 3, 1, 3], [2, 4, 6, 12]
    coef = m.predictor_fit(n, L, t)
    assert np.allclose(coef, g["ols_coef"], atol=1e-12)
    assert abs(m.mape_pct(coef, n, L, t) - g["ols_mape_pct"][0]) < 1e-9


def pin_exact_recovery_on_the_paper_grid(m):
    c = {k: v for k, v in (line.split("#")[0].split() for line in open(os.path.join(G, "paper_constants.txt"))
                           if len(line.split("#")[0].split()) == 2)}
    nb, nc = int(c["predictor_grid_batches"]), int(c["predictor_grid_contexts"])
    assert nb * nc == int(c["predictor_profile_steps"])
    batches = np.unique(np.round(np.geomspace(1, float(c["predictor_batch_max"]), nb)))
    ctxs = np.linspace(float(c["predictor_context_min"]), float(c["predictor_context_max"]), nc)
    n, L = np.meshgrid(batches, ctxs, indexing="ij")
    n, L = n.ravel(), (n * L).ravel()  # aggregate context = batch x per-sequence context
    true = (0.37, 0.0123, 4.56e-6)
    t = true[0] + true[1] * n + true[2] * L
    coef = m.predictor_fit(n, L, t)
    assert np.allclose(coef, true, rtol=1e-9)
    assert m.mape_pct(coef, n, L, t) < 1e-9
    assert m.predictor_eval(coef, 7, 9000) == pytest.approx(0.37 + 0.0123 * 7 + 4.56e-6 * 9000, rel=1e-12)


def pin_residual_is_orthogonal_to_the_regressors(m):
    rng = np.random.default_rng(5)
    n = rng.integers(1, 513, 300).astype(float)
    L = n * rng.integers(128, 8193, 300)
    t = 0.2 + 0.01 * n + 3e-6 * L + rng.normal(0, 0.05, 300)
    a, b, c = m.predictor_fit(n, L, t)
    r = t - (a + b * n + c * L)
    for x in (np.ones_like(n), n, L):
        assert abs(np.dot(r, x)) <= 1e-7 * np.linalg.norm(x) * np.linalg.norm(t)
    # any other coefficients have a larger residual
    for d in ((1e-3, 0, 0), (0, 1e-5, 0), (0, 0, 1e-9)):
        r2 = t - ((a + d[0]) + (b + d[1]) * n + (c + d[2]) * L)
        assert np.dot(r2, r2) > np.dot(r, r)


def pin_mape_definition(m):
    # predictions 110 and 90 against observations 100 and 100 -> 10 %; against 50 and 100 -> (120 % + 10 %) / 2
    coef = (0.0, 1.0, 0.0)
    assert m.mape_pct(coef, [110, 90], [0, 0], [100, 100]) == pytest.approx(10.0)
    assert m.mape_pct(coef, [110, 90], [0, 0], [50, 100]) == pytest.approx(65.0)


def pin_rolling_window_forgets_old_steps(m):
    old = [(n, n * 100, 5.0 + 1.0 * n + 0.01 * n * 100 + (n % 3)) for n in range(1, 120)]
    new = [(n, n * (50 + n % 7), 1.0 + 0.5 * n + 0.002 * n * (50 + n % 7)) for n in range(1, 201)]
    assert np.allclose(m.rolling_fit(old + new, window=200), (1.0, 0.5, 0.002), rtol=1e-8)


# ---------------------------------------------------------------- planner pins
def pin_budget_formula(m):
    assert m.slack_budget(10.0, 30.0, 0.5) == pytest.approx(20.0)
    assert m.slack_budget(10.0, 30.0, 1.0) == pytest.approx(30.0)
    assert m.slack_budget(10.0, 7.0, 0.9) == 10.0  # no residual: B_t = 0


def pin_worked_example(m):
    g = golden()
    for case, reqs, rho in (("A", example_requests(m), 0.5), ("B", example_requests(m, slack0=8.0), 0.5),
                            ("C", example_requests(m), 1.0)):
        p = m.taper_step(reqs, COEF, rho)
        assert p.budget == pytest.approx(g[case + "_budget"][0], abs=1e-12), case
        assert p.granted == [int(x) for x in g[case + "_granted"]], case
        assert p.t_pred == pytest.approx(g[case + "_t_pred"][0], abs=1e-9), case
    p = m.taper_step(example_requests(m), COEF, 0.5)
    assert (p.n_tokens, p.l_context, p.evaluations) == (g["A_n_tokens"][0], g["A_l_context"][0], g["A_evaluations"][0])
    assert p.t0 == pytest.approx(4.8)
    assert m.taper_step(example_requests(m, slack0=8.0), COEF, 0.5).evaluations == g["B_evaluations"][0]  # pruning is for good


def random_requests(m, rng, n_req, kind="linear"):
    reqs = []
    for _ in range(n_req):
        base = int(rng.integers(100, 3000))
        nb = int(rng.integers(0, 4))
        w = float(rng.integers(1, 4))
        reqs.append(m.Request(base, float(rng.uniform(5, 40)), [base + int(rng.integers(0, 500)) for _ in range(nb)],
                              m.utility_curve(kind, w)))
    return reqs


def pin_feasible_and_maximal_against_brute_force(m):
    """On tiny inputs enumerate every grant vector: the greedy result is feasible, and it
    is maximal (no single further branch fits) -- with increasing utilities the loop may
    only stop for lack of a feasible increment."""
    rng = np.random.default_rng(11)
    T = lambda n, L: COEF[0] + COEF[1] * n + COEF[2] * L
    for trial in range(60):
        reqs = random_requests(m, rng, int(rng.integers(1, 5)), kind=("linear", "concave")[trial % 2])
        rho = float(rng.uniform(0.1, 1.0))
        p = m.taper_step(reqs, COEF, rho)
        n0, L0 = len(reqs), sum(r.base_context for r in reqs)
        t0 = T(n0, L0)
        budget = t0 + rho * max(0.0, min(r.slack_ms for r in reqs) - t0)
        assert p.budget == pytest.approx(budget, rel=1e-12) and p.t0 == pytest.approx(t0, rel=1e-12)

        def t_of(gv):
            return T(n0 + sum(gv), L0 + sum(sum(r.branch_context[:k]) for r, k in zip(reqs, gv)))

        assert t_of(p.granted) <= budget + 1e-12
        assert p.t_pred == pytest.approx(t_of(p.granted), rel=1e-12)
        assert all(0 <= k <= len(r.branch_context) for r, k in zip(reqs, p.granted))
        feasible = [gv for gv in itertools.product(*[range(len(r.branch_context) + 1) for r in reqs]) if t_of(gv) <= budget]
        assert tuple(p.granted) in feasible
        for i, r in enumerate(reqs):
            if p.granted[i] < len(r.branch_context):
                gv = list(p.granted)
                gv[i] += 1
                assert t_of(gv) > budget, "a further branch would still fit"


def pin_no_slack_no_width_and_ample_slack_full_width(m):
    reqs = example_requests(m)
    reqs[0].slack_ms = 4.0  # below T0 = 4.8
    assert m.taper_step(reqs, COEF, 1.0).granted == [0, 0, 0]
    reqs = example_requests(m)
    for r in reqs:
        r.slack_ms = 1e6
    assert m.taper_step(reqs, COEF, 0.01).granted == [0, 3, 2]


def pin_equal_branches_closed_form(m):
    """Identical branch cost d = b + c ctx: exactly floor((budget - T0) / d) branches are admitted."""
    lin = m.utility_curve("linear", 1.0)
    ctx = 1000
    reqs = [m.Request(ctx, 31.7, [ctx] * 6, lin) for _ in range(4)]
    p = m.taper_step(reqs, COEF, 0.8)
    d = COEF[1] + COEF[2] * ctx
    assert sum(p.granted) == math.floor((p.budget - p.t0) / d + 1e-9)
    assert 0 < sum(p.granted) < 24
    # concave utility spreads the same number evenly
    con = m.utility_curve("concave", 1.0)
    reqs = [m.Request(ctx, 31.7, [ctx] * 6, con) for _ in range(4)]
    q = m.taper_step(reqs, COEF, 0.8)
    assert sum(q.granted) == sum(p.granted) and max(q.granted) - min(q.granted) <= 1
    # linear utility, equal scores: the earlier request keeps winning the tie
    assert p.granted == sorted(p.granted, reverse=True) and p.granted[0] == 6


def pin_cheapest_first_under_linear_utility(m):
    """Equal marginal utility: the branch with the smallest marginal latency goes first, so with a
    budget for exactly one branch the request with the shortest branch gets it."""
    lin = m.utility_curve("linear", 1.0)
    reqs = [m.Request(1000, 1e3, [5000], lin), m.Request(1000, 1e3, [300], lin), m.Request(1000, 1e3, [4000], lin)]
    t0 = COEF[0] + COEF[1] * 3 + COEF[2] * 3000
    for r in reqs:
        r.slack_ms = t0 + 1.0  # residual 1 ms, rho 1: only the 0.4 ms branch fits
    assert m.taper_step(reqs, COEF, 1.0).granted == [0, 1, 0]
    # weight can outvote cost: a heavy request with a dearer branch wins when both fit
    reqs = [m.Request(1000, 1e3, [2000], m.utility_curve("linear", 10.0)), m.Request(1000, 1e3, [300], lin)]
    t0 = COEF[0] + COEF[1] * 2 + COEF[2] * 2000
    for r in reqs:
        r.slack_ms = t0 + 2.2  # 2.1 fits, 2.1 + 0.4 does not
    assert m.taper_step(reqs, COEF, 1.0).granted == [1, 0]


def pin_table_utility_and_zero_gain_stops(m):
    flat = m.utility_curve("table", table=[0.0, 1.0, 1.0, 1.0])  # nothing gained after the first branch
    reqs = [m.Request(1000, 1e6, [1000, 1000, 1000], flat)]
    assert m.taper_step(reqs, COEF, 1.0).granted == [1]


def _kkt(coef, n, L, t):
    """Optimality of a fit over the region b, c >= 0: the gradient of the squared error vanishes along the
    free coordinates and points into the region along the clamped ones."""
    n, L, t = (np.asarray(x, np.float64) for x in (n, L, t))
    res = coef[0] + coef[1] * n + coef[2] * L - t
    g = np.array([res.sum(), (res * n).sum(), (res * L).sum()])
    scale = np.array([len(t), np.abs(n).sum(), np.abs(L).sum()]) * np.abs(t).max()
    assert abs(g[0]) <= 1e-9 * scale[0]
    for k in (1, 2):
        assert coef[k] >= 0
        if coef[k] > 0:
            assert abs(g[k]) <= 1e-9 * scale[k]
        else:
            assert g[k] >= -1e-9 * scale[k]


def pin_monotone_fit_equals_ols_inside_the_region(m):
    rng = np.random.default_rng(5)
    n = rng.integers(1, 512, 60).astype(float)
    L = n * rng.integers(128, 8192, 60)
    t = 0.04 + 1e-4 * n + 2.4e-6 * L + rng.normal(0, 1e-3, 60)
    assert np.allclose(m.predictor_fit_monotone(n, L, t), m.predictor_fit(n, L, t), rtol=1e-7, atol=1e-12)


def pin_monotone_fit_clamps_and_refits(m):
    """Steps whose time falls with the batch size (launch-bound, noisy): the slope on n_tokens would be
    negative.  The constrained fit puts it at exactly 0 and the rest is the line in L_context alone."""
    n = np.array([1, 1, 1, 1, 4, 4, 4, 4, 16, 16, 16, 16, 64, 64, 64, 64], float)
    c = np.array([128, 1024, 4096, 8192] * 4, float)
    L = n * c
    t = 0.03 + 1.2e-6 * L - 3.2e-4 * n  # what a 16-point probe run once produced: b < 0
    free = m.predictor_fit(n, L, t)
    assert free[1] < 0
    a, b, cc = m.predictor_fit_monotone(n, L, t)
    assert b == 0.0 and cc > 0
    slope, icpt = np.polyfit(L, t, 1)
    assert a == pytest.approx(icpt, rel=1e-9) and cc == pytest.approx(slope, rel=1e-9)
    _kkt((a, b, cc), n, L, t)
    # both slopes negative: the mean
    t2 = 5.0 - 1e-3 * n - 1e-7 * L
    a, b, cc = m.predictor_fit_monotone(n, L, t2)
    assert b == 0.0 and cc == 0.0 and a == pytest.approx(t2.mean(), rel=1e-12)


def pin_monotone_fit_is_the_constrained_minimum(m):
    rng = np.random.default_rng(6)
    for trial in range(20):
        n = rng.integers(1, 64, 16).astype(float)
        L = n * rng.integers(128, 8192, 16)
        t = 0.05 + rng.normal(0, 2e-4) * n + rng.normal(1e-6, 2e-6) * L + rng.normal(0, 5e-3, 16)
        coef = np.array(m.predictor_fit_monotone(n, L, t))
        _kkt(coef, n, L, t)
        rss = lambda c: float(((c[0] + c[1] * n + c[2] * L - t) ** 2).sum())
        best = rss(coef)
        for _ in range(200):  # no feasible point nearby does better
            d = rng.normal(0, 1, 3) * np.array([1e-3, 1e-5, 1e-8])
            cand = coef + d
            cand[1:] = np.maximum(cand[1:], 0.0)
            assert rss(cand) >= best * (1 - 1e-12)


PINS = [pin_monotone_fit_equals_ols_inside_the_region, pin_monotone_fit_clamps_and_refits,
        pin_monotone_fit_is_the_constrained_minimum, pin_ols_by_hand, pin_exact_recovery_on_the_paper_grid, pin_residual_is_orthogonal_to_the_regressors,
        pin_mape_definition, pin_rolling_window_forgets_old_steps, pin_budget_formula, pin_worked_example,
        pin_feasible_and_maximal_against_brute_force, pin_no_slack_no_width_and_ample_slack_full_width,
        pin_equal_branches_closed_form, pin_cheapest_first_under_linear_utility, pin_table_utility_and_zero_gain_stops]


@pytest.mark.parametrize("pin", PINS, ids=lambda f: f.__name__)
def test_pin(pin):
    pin(load_module())


MUTANTS = {
    "regressors_swapped": ("X = np.stack([np.ones_like(n), n, L], axis=1)", "X = np.stack([np.ones_like(n), L, n], axis=1)"),
    "no_intercept": ("X = np.stack([np.ones_like(n), n, L], axis=1)", "X = np.stack([np.zeros_like(n), n, L], axis=1)"),
    "mape_relative_to_prediction": ("np.abs(pred - t) / np.abs(t)", "np.abs(pred - t) / np.abs(pred)"),
    "window_takes_oldest": ("obs = list(observations)[-window:]", "obs = list(observations)[:window]"),
    "budget_forgets_baseline": ("rho * max(0.0, min_slack - t0)", "rho * max(0.0, min_slack)"),
    "budget_ignores_rho": ("return t0 + rho * max(0.0, min_slack - t0)", "return t0 + max(0.0, min_slack - t0)"),
    "slack_of_the_richest_request": ("min(r.slack_ms for r in requests)", "max(r.slack_ms for r in requests)"),
    "slack_only_of_requests_with_branches": ("min(r.slack_ms for r in requests)",
                                             "min(r.slack_ms for r in requests if r.branch_context)"),
    "feasibility_on_increment_only": ("if priced[i] <= budget]", "if priced[i] - t_step <= budget]"),
    "branch_priced_as_its_parent": ("step[1] + requests[i].branch_context[granted[i]]", "step[1] + requests[i].base_context"),
    "always_first_branch_context": ("step[1] + requests[i].branch_context[granted[i]]", "step[1] + requests[i].branch_context[0]"),
    "token_count_not_widened": ("return (step[0] + 1, step[1]", "return (step[0], step[1]"),
    "score_ignores_cost": ("return gain / (EPS + max(0.0, t_widened - t_step))", "return gain"),
    "score_ignores_utility": ("return gain / (EPS + max(0.0, t_widened - t_step))", "return 1.0 / (EPS + max(0.0, t_widened - t_step))"),
    "later_request_wins_ties": ("chosen = feasible[ratios.index(top)]", "chosen = feasible[len(ratios) - 1 - ratios[::-1].index(top)]"),
    "pruned_request_comes_back": ("considered = [i for i in feasible if granted[i]", "considered = [i for i in considered if granted[i]"),
    "stops_one_branch_early": ("if granted[i] < len(requests[i].branch_context)]",
                               "if granted[i] < len(requests[i].branch_context) - 1]"),
    "monotone_fit_forgets_a_bound": ("bounds=([-np.inf, 0.0, 0.0]", "bounds=([-np.inf, -np.inf, 0.0]"),
    "monotone_fit_bounds_the_intercept": ("bounds=([-np.inf, 0.0, 0.0]", "bounds=([0.0, 0.0, 0.0]"),
    "concave_is_linear": ("return lambda k: weight * math.log2(1.0 + k)", "return lambda k: weight * k"),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_reject_mutant(name):
    old, new = MUTANTS[name]
    src = open(SRC).read()
    assert src.count(old) == 1, f"mutation site for {name} not found exactly once"
    m = load_module(src.replace(old, new), name="admission_mutant_" + name)
    failed = []
    for pin in PINS:
        try:
            pin(m)
        except Exception as e:  # noqa: BLE001 - any failure of a pin counts
            failed.append(pin.__name__)
    assert failed, f"mutant {name} slipped through every pin"
