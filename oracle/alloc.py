"""CPU oracle for the bit-width allocation (test infrastructure only: the tests import this, the product never does).

Sec. 3.3, Eq. 2: every layer i picks exactly one candidate bit-width b; the pick maximises the summed sensitivity
score S[i][b] subject to the summed resource cost M[i][b] staying within the budget B.  The first function is that
definition written out (all assignments are enumerated); the second is the textbook dynamic programme over integer
costs for instances too large to enumerate, pinned against the first by the tests.  App. A, Alg. 1 wraps the
integer programme in two loops (M budgets below the target, N content/quality ratios); the image generation and
scoring at the end of each iteration need the model and are not part of this code: the candidate configurations are
returned for the caller to score.

Plain Python and numpy, float64 sums in layer order.
"""
from __future__ import annotations

import itertools
import math

import numpy as np


def objective(sens, choice) -> float:
    """Sum of the chosen sensitivity scores, added in layer order (Eq. 2's objective)."""
    total = 0.0
    for i, c in enumerate(choice):
        total += float(sens[i][c])
    return total


def total_cost(cost, choice) -> int:
    return sum(int(cost[i][c]) for i, c in enumerate(choice))


def allocate_bruteforce(sens, cost, budget):
    """Eq. 2 by enumeration.  sens, cost: [n_layers][n_choices]; budget: int.
    Returns (best objective, one maximising choice tuple), or None when no assignment fits the budget."""
    n = len(sens)
    m = len(sens[0])
    best = None
    for choice in itertools.product(range(m), repeat=n):
        if total_cost(cost, choice) > budget:
            continue
        v = objective(sens, choice)
        if best is None or v > best[0]:
            best = (v, choice)
    return best


def allocate_dp(sens, cost, budget):
    """Eq. 2 by the multiple-choice knapsack recurrence over integer costs:
        best_i[c] = max_b  best_{i-1}[c - M[i][b]] + S[i][b]          (c = total cost so far, exactly)
    Costs are divided by their common divisor first (every reachable total is a multiple of it).
    Returns (objective, choice tuple) or None when infeasible."""
    sens = np.asarray(sens, np.float64)
    cost = np.asarray(cost, np.int64)
    n, m = sens.shape
    g = 0
    for v in cost.ravel():
        g = math.gcd(g, int(v))
    g = max(g, 1)
    units = cost // g
    cap = int(budget) // g
    if cap < 0:
        return None
    NEG = -np.inf
    best = np.full(cap + 1, NEG)
    best[0] = 0.0
    pick = np.zeros((n, cap + 1), np.int8)
    for i in range(n):
        new = np.full(cap + 1, NEG)
        for b in range(m):
            u = int(units[i, b])
            if u > cap:
                continue
            cand = np.full(cap + 1, NEG)
            cand[u:] = best[:cap + 1 - u] + sens[i, b]
            better = cand > new
            new[better] = cand[better]
            pick[i, better] = b
        best = new
    if not np.isfinite(best).any():
        return None
    c = int(np.argmax(best))          # first (cheapest) total cost that reaches the maximum
    value = float(best[c])
    choice = [0] * n
    for i in range(n - 1, -1, -1):
        b = int(pick[i, c])
        choice[i] = b
        c -= int(units[i, b])
    assert c == 0
    return value, tuple(choice)


def layer_costs(params, bits):
    """M[i][b] = P_i * b: the budget is stated as an average bit-width over all elements (Sec. 4.1, "Mixed
    Precision Allocation"), so a layer costs its element count times its bit-width."""
    return [[int(p) * int(b) for b in bits] for p in params]


def split_budget(b_all: int, p_content: int, p_quality: int, k: float):
    """App. A, Alg. 1, SplitBudget.  The paper defines K only as the ratio in which the budget is shared between the
    content group and the quality group, and scans values near one.  Reading taken: K is the ratio of the two groups'
    average bit-widths, avg_content = K * avg_quality, with B_content + B_quality = B_all.
    Returns (B_content, B_quality) in bits; B_content is rounded down, the rest goes to the quality group."""
    avg_q = b_all / (k * p_content + p_quality)
    b_content = int(math.floor(k * avg_q * p_content))
    return b_content, int(b_all) - b_content


def search_candidates(sens_c, params_c, sens_q, params_q, bits, avg_bits_target, delta_avg_bits, n_budgets, k_lo, k_hi,
                      n_ratios, solver=allocate_dp):
    """App. A, Alg. 1 without its last two steps (generation and scoring of images): for each of n_budgets budgets
    spaced linearly in [B_all - dB, B_all] and each of n_ratios ratios spaced linearly in [k_lo, k_hi], split the
    budget, solve Eq. 2 for each group, and join the two configurations.
    B_all = avg_bits_target * (P_content + P_quality), dB = delta_avg_bits * (P_content + P_quality), rounded down.
    Returns a list of dicts (budget, k, b_content, b_quality, feasible, objective_c, objective_q, choice_c, choice_q)."""
    pc, pq = int(sum(params_c)), int(sum(params_q))
    b_all = int(math.floor(avg_bits_target * (pc + pq)))
    d_b = int(math.floor(delta_avg_bits * (pc + pq)))
    cost_c, cost_q = layer_costs(params_c, bits), layer_costs(params_q, bits)
    out = []
    for j in range(n_budgets):
        frac = j / (n_budgets - 1) if n_budgets > 1 else 1.0
        bj = b_all - d_b + int(math.floor(frac * d_b))
        for t in range(n_ratios):
            k = k_lo + (k_hi - k_lo) * (t / (n_ratios - 1) if n_ratios > 1 else 0.0)
            bc, bq = split_budget(bj, pc, pq, k)
            rc = solver(sens_c, cost_c, bc)
            rq = solver(sens_q, cost_q, bq)
            ok = rc is not None and rq is not None
            out.append(dict(budget=bj, k=k, b_content=bc, b_quality=bq, feasible=ok,
                            objective_c=rc[0] if ok else None, objective_q=rq[0] if ok else None,
                            choice_c=rc[1] if ok else None, choice_q=rq[1] if ok else None))
    return out
