"""CPU oracle for the controller side of the paper: the latency predictor of App. C
("Predictor formulation", "Fitting") and the per-step admission of §3.3 (slack
budget) and §3.4 (greedy planner).  Test infrastructure only: plain, slow,
float64; nothing in the product imports it.

Readings taken where the paper leaves a choice (each also listed in the design notes):
  * the composition S is the pair (n_tokens, L_context) of App. C; AddBranch adds
    one token and the context length of the request's next ready branch, branches
    of a request being admitted in the order the caller lists them;
  * requests are scanned in increasing index; on equal score the earlier one wins
    (the listing keeps the first best and replaces it only on a strictly larger score);
  * EPS of the score's denominator is 1e-9 (milliseconds);
  * utility curves: "linear" u(k) = w k, "concave" u(k) = w log2(1 + k) (first
    opportunistic branch worth w, later ones less), or a caller-supplied table.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Callable, List, Optional, Sequence

import numpy as np

EPS = 1e-9


# ----------------------------------------------------------------------------- App. C
def predictor_fit(n_tokens, l_context, t_ms):
    """Ordinary least squares for T = a + b n_tokens + c L_context (App. C, "Fitting").
    The library routine is the definition: minimise ||X beta - t||_2, X = [1, n, L]."""
    n = np.asarray(n_tokens, np.float64)
    L = np.asarray(l_context, np.float64)
    t = np.asarray(t_ms, np.float64)
    X = np.stack([np.ones_like(n), n, L], axis=1)
    beta, _, rank, _ = np.linalg.lstsq(X, t, rcond=None)
    if rank < 3:
        raise ValueError("observations do not determine (a, b, c)")
    return float(beta[0]), float(beta[1]), float(beta[2])


def predictor_fit_monotone(n_tokens, l_context, t_ms):
    """The fit under b >= 0, c >= 0 (App. C, "Monotonicity": T must be monotone in admitted branches).
    Definition: minimise ||X beta - t||_2 over that region; the library's bounded least squares is the step
    (columns scaled to unit max so that its tolerances mean the same for both regressors)."""
    from scipy.optimize import lsq_linear

    n = np.asarray(n_tokens, np.float64)
    L = np.asarray(l_context, np.float64)
    t = np.asarray(t_ms, np.float64)
    sn, sL = np.abs(n).max(), np.abs(L).max()
    X = np.stack([np.ones_like(n), n / sn, L / sL], axis=1)
    r = lsq_linear(X, t, bounds=([-np.inf, 0.0, 0.0], [np.inf, np.inf, np.inf]), method="bvls", tol=1e-14)
    return float(r.x[0]), float(r.x[1] / sn), float(r.x[2] / sL)


def predictor_eval(coef, n_tokens, l_context):
    a, b, c = coef
    return a + b * n_tokens + c * l_context


def mape_pct(coef, n_tokens, l_context, t_ms):
    """Mean absolute percentage error of the predictor over the observations (App. C, "Accuracy")."""
    t = np.asarray(t_ms, np.float64)
    pred = predictor_eval(coef, np.asarray(n_tokens, np.float64), np.asarray(l_context, np.float64))
    return float(np.mean(np.abs(pred - t) / np.abs(t)) * 100.0)


def rolling_fit(observations, window=200):
    """Refresh of App. C: the fit over the most recent `window` observed steps."""
    obs = list(observations)[-window:]
    return predictor_fit([o[0] for o in obs], [o[1] for o in obs], [o[2] for o in obs])


# ----------------------------------------------------------------------------- §3.3
def slack_budget(t0, min_slack, rho):
    """Largest admissible predicted step latency: T0 + rho * B_t with
    B_t = max(0, min_r (d_r - t) - T0)  (§3.3)."""
    return t0 + rho * max(0.0, min_slack - t0)


def utility_curve(kind: str, weight: float = 1.0, table: Optional[Sequence[float]] = None) -> Callable[[int], float]:
    if kind == "linear":
        return lambda k: weight * k
    if kind == "concave":
        return lambda k: weight * math.log2(1.0 + k)
    if kind == "table":
        tab = list(table)
        return lambda k: tab[k]
    raise ValueError(kind)


# ----------------------------------------------------------------------------- §3.4
@dataclass
class Request:
    base_context: int                 # context length of the request's protected continuation (one token in S_0)
    slack_ms: float                   # d_r(t) - t
    branch_context: List[int]         # context lengths of its ready branches, in admission order
    utility: Callable[[int], float]   # u_r(k), k = opportunistic branches granted


@dataclass
class StepPlan:
    granted: List[int]
    n_tokens: int
    l_context: int
    t0: float
    budget: float
    t_pred: float
    evaluations: int                  # calls of T made while widening


def taper_step(requests: Sequence[Request], coef, rho: float) -> StepPlan:
    """Per-step admission as the definitions state it (§3.3, §3.4).

    The step starts as the protected composition S_0 and is widened one branch at a time.  In every round:
      1. feasibility (§3.3): of the requests still under consideration, those whose widened step would keep
         T(S) within the budget T_0 + rho * B_t form the feasible set; the others leave for good (T is
         monotone in admitted branches, so nothing of theirs can fit later);
      2. selection (§3.4): among the feasible ones the branch with the largest marginal utility per marginal
         predicted latency is admitted -- unless that best ratio is not positive, or nothing is feasible,
         which ends the step.
    A request with no ready branch left is no longer under consideration."""
    T = lambda comp: predictor_eval(coef, comp[0], comp[1])
    step = (len(requests), sum(r.base_context for r in requests))  # (n_tokens, L_context) of S_0
    t0 = T(step)
    budget = slack_budget(t0, min(r.slack_ms for r in requests), rho)
    granted = [0] * len(requests)
    considered = [i for i, r in enumerate(requests) if r.branch_context]
    t_step, evaluations = t0, 0

    def widened(i):
        return (step[0] + 1, step[1] + requests[i].branch_context[granted[i]])

    def ratio(i, t_widened):
        gain = requests[i].utility(granted[i] + 1) - requests[i].utility(granted[i])
        return gain / (EPS + max(0.0, t_widened - t_step))

    while considered:
        priced = {i: T(widened(i)) for i in considered}  # one evaluation of T per request and round
        evaluations += len(priced)
        feasible = [i for i in considered if priced[i] <= budget]
        if not feasible:
            break
        ratios = [ratio(i, priced[i]) for i in feasible]
        top = max(ratios)
        if top <= 0:
            break
        chosen = feasible[ratios.index(top)]  # the earliest request among equals
        step, t_step = widened(chosen), priced[chosen]
        granted[chosen] += 1
        considered = [i for i in feasible if granted[i] < len(requests[i].branch_context)]
    return StepPlan(granted, step[0], step[1], t0, budget, t_step, evaluations)
