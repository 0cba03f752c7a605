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
    """Greedy widening of the protected composition (§3.4): repeatedly admit the ready
    branch with the best marginal utility per marginal predicted latency among those
    whose widened step still fits the slack budget; a request whose next branch does
    not fit is dropped for good (T is monotone)."""
    T = lambda n, L: predictor_eval(coef, n, L)
    n = len(requests)
    L = sum(r.base_context for r in requests)
    t0 = T(n, L)
    budget = slack_budget(t0, min(r.slack_ms for r in requests), rho)
    granted = [0] * len(requests)
    live = [i for i, r in enumerate(requests) if len(r.branch_context) > 0]
    t_step = t0
    evals = 0
    while live:
        best = None
        still = []
        for i in live:
            r = requests[i]
            n_w, L_w = n + 1, L + r.branch_context[granted[i]]
            t_w = T(n_w, L_w)
            evals += 1
            if t_w > budget:
                continue  # pruned: no later branch of r can fit either
            still.append(i)
            du = r.utility(granted[i] + 1) - r.utility(granted[i])
            score = du / (EPS + max(0.0, t_w - t_step))
            if best is None or score > best[0]:
                best = (score, i, n_w, L_w, t_w)
        live = still
        if best is None or best[0] <= 0:
            break
        _, i, n, L, t_step = best
        granted[i] += 1
        if granted[i] >= len(requests[i].branch_context):
            live.remove(i)
    return StepPlan(granted, n, L, t0, budget, t_step, evals)
