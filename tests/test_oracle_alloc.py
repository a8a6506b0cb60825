"""Pins of the bit-width allocation oracle (CPU): Eq. 2 by enumeration against hand-worked cases, a textbook knapsack,
closed forms and invariants; the dynamic programme against the enumeration; the budget split and the candidate scan."""
import itertools
import math

import numpy as np
import pytest

import synth_inputs as si
from oracle import alloc


def test_hand_worked_three_layers():
    """Three layers, bits {2,4,8}, elements P = (10, 20, 5), costs P*b = [[20,40,80],[40,80,160],[10,20,40]],
        S = [[1, 5, 6], [1, 3, 9], [0, 4, 5]].
    Budget 170.  Layer 1 at 8 bits needs 160 + 20 + 10 = 190: out.  Without it the best conceivable score is
    6 + 3 + 5 = 14 at 8/4/8 bits, cost 200: out.  One step down from there: 4/4/8 costs 160 and scores 13;
    8/2/8 costs 160 and scores 12; 8/4/4 costs 180: out; so 13 at (4, 4, 8) bits, and no other assignment reaches 13.
    Budget 220 admits 4/8/4 bits (40 + 160 + 20): 5 + 9 + 4 = 18, against 2/8/8 (220): 15 and 8/4/8 (200): 14."""
    S = [[1, 5, 6], [1, 3, 9], [0, 4, 5]]
    cost = alloc.layer_costs([10, 20, 5], (2, 4, 8))
    assert cost == [[20, 40, 80], [40, 80, 160], [10, 20, 40]]
    assert alloc.allocate_bruteforce(S, cost, 170) == (13.0, (1, 1, 2))
    assert alloc.allocate_dp(S, cost, 170) == (13.0, (1, 1, 2))
    assert alloc.allocate_bruteforce(S, cost, 220) == (18.0, (1, 2, 1))
    assert alloc.allocate_dp(S, cost, 220) == (18.0, (1, 2, 1))
    # the budget is an upper bound, not a target: at 219 layer 1 at 8 bits leaves 59 for the others (2/8/4 or 4/8/2
    # bits, 14 either way), which ties with 8/4/8
    assert alloc.allocate_bruteforce(S, cost, 219)[0] == 14.0 and alloc.allocate_dp(S, cost, 219)[0] == 14.0
    # the cheapest assignment costs 70, everything at 8 bits 280
    assert alloc.allocate_bruteforce(S, cost, 69) is None and alloc.allocate_dp(S, cost, 69) is None
    assert alloc.allocate_bruteforce(S, cost, 70) == (2.0, (0, 0, 0))
    assert alloc.allocate_bruteforce(S, cost, 280) == (20.0, (2, 2, 2))
    assert alloc.allocate_dp(S, cost, 10 ** 4) == (20.0, (2, 2, 2))


def test_reduces_to_the_textbook_01_knapsack():
    """Two choices per layer, the first free and worthless: Eq. 2 becomes the 0/1 knapsack.  The classic instance
    weights (1, 3, 4, 5), values (1, 4, 5, 7), capacity 7 has optimum 9 (items of weight 3 and 4)."""
    w, val = (1, 3, 4, 5), (1, 4, 5, 7)
    S = [[0, v] for v in val]
    cost = [[0, x] for x in w]
    assert alloc.allocate_bruteforce(S, cost, 7) == (9.0, (0, 1, 1, 0))
    assert alloc.allocate_dp(S, cost, 7) == (9.0, (0, 1, 1, 0))
    # a transposed table (choices x layers) or a swapped sens/cost would not reproduce 9 with this choice
    assert alloc.allocate_dp(cost, S, 7)[1] != (0, 1, 1, 0)


@pytest.mark.parametrize("seed", range(12))
def test_dp_equals_enumeration_on_random_instances(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 8))
    m = int(rng.integers(2, 5))
    params = rng.integers(1, 30, n) * int(rng.choice([1, 4, 64]))
    bits = sorted(rng.choice(np.arange(1, 17), m, replace=False).tolist())
    cost = alloc.layer_costs(params, bits)
    if seed % 3 == 0:
        S = rng.integers(0, 6, (n, m)).astype(np.float64)      # many ties
    else:
        S = rng.normal(0, 10, (n, m))                            # not monotone in b: Eq. 2 does not need it
    lo = sum(min(r) for r in cost)
    hi = sum(max(r) for r in cost)
    for budget in {lo - 1, lo, (lo + hi) // 2, (2 * lo + hi) // 3, hi - 1, hi, hi + 5}:
        bf = alloc.allocate_bruteforce(S, cost, budget)
        dp = alloc.allocate_dp(S, cost, budget)
        if bf is None:
            assert dp is None
            continue
        assert dp[0] == bf[0], (budget, dp, bf)        # same additions in the same order: equal to the last bit
        assert alloc.total_cost(cost, dp[1]) <= budget
        assert alloc.objective(S, dp[1]) == dp[0]


def test_invariants_monotone_in_the_budget_and_closed_forms():
    n = 9
    S = si.sensitivity_table(3, "pin/alloc", n)
    params = [320 * 320, 640 * 640, 2048 * 640, 9 * 320 * 320, 1280 * 1280, 640 * 5120, 2560 * 640, 320, 640 * 640]
    cost = alloc.layer_costs(params, (2, 4, 8))
    P = sum(params)
    prev = -math.inf
    for avg in np.linspace(2.0, 8.0, 13):
        r = alloc.allocate_dp(S, cost, int(avg * P))
        assert r is not None and r[0] >= prev
        prev = r[0]
        assert alloc.total_cost(cost, r[1]) <= int(avg * P)
        assert r[0] == alloc.allocate_bruteforce(S, cost, int(avg * P))[0]
    assert alloc.allocate_dp(S, cost, 2 * P)[1] == (0,) * n              # only the all-2-bit assignment fits
    assert alloc.allocate_dp(S, cost, 8 * P)[1] == (2,) * n              # scores rise with b: all 8 bit
    assert alloc.allocate_dp(S, cost, 2 * P - 1) is None
    # weak duality: for every multiplier lam >= 0,  OPT <= sum_i max_b (S - lam*M) + lam*B
    B = int(4.5 * P)
    opt = alloc.allocate_dp(S, cost, B)[0]
    C = np.asarray(cost, np.float64)
    for lam in np.linspace(0, 1e-4, 200):
        assert opt <= (S - lam * C).max(1).sum() + lam * B + 1e-9


def test_budget_split_and_candidate_scan():
    # K = 1: both groups get the same average bit-width
    bc, bq = alloc.split_budget(5 * 300, 100, 200, 1.0)
    assert (bc, bq) == (500, 1000)
    # K = 2: content average twice the quality average, budgets add up:  a_q = 1500 / (2*100 + 200) = 3.75
    bc, bq = alloc.split_budget(1500, 100, 200, 2.0)
    assert (bc, bq) == (750, 750) and bc / 100 == 2.0 * bq / 200
    for k in (0.45, 0.9, 1.36):
        bc, bq = alloc.split_budget(123457, 1000, 777, k)
        assert bc + bq == 123457 and abs((bc / 1000) / (bq / 777) - k) < 1e-3
    rng = np.random.default_rng(5)
    pc, pq = [64, 128, 64, 256], [32, 32, 512]
    sc, sq = si.sensitivity_table(5, "pin/sc", 4), si.sensitivity_table(5, "pin/sq", 3)
    cands = alloc.search_candidates(sc, pc, sq, pq, (2, 4, 8), 5.0, 1.0, 3, 0.5, 1.5, 4)
    assert len(cands) == 12
    P = sum(pc) + sum(pq)
    assert [c["budget"] for c in cands[::4]] == [4 * P, 4 * P + P // 2, 5 * P]
    assert [round(c["k"], 6) for c in cands[:4]] == [0.5, round(0.5 + 1 / 3, 6), round(0.5 + 2 / 3, 6), 1.5]
    for c in cands:
        assert c["b_content"] + c["b_quality"] == c["budget"]
        if c["feasible"]:
            cc, cq = alloc.layer_costs(pc, (2, 4, 8)), alloc.layer_costs(pq, (2, 4, 8))
            assert alloc.total_cost(cc, c["choice_c"]) <= c["b_content"]
            assert alloc.total_cost(cq, c["choice_q"]) <= c["b_quality"]
            assert c["objective_c"] == alloc.allocate_bruteforce(sc, cc, c["b_content"])[0]
            assert c["objective_q"] == alloc.allocate_bruteforce(sq, cq, c["b_quality"])[0]
    assert any(c["feasible"] for c in cands)
    # with the brute-force solver plugged in the scan returns the same objectives
    again = alloc.search_candidates(sc, pc, sq, pq, (2, 4, 8), 5.0, 1.0, 3, 0.5, 1.5, 4, solver=alloc.allocate_bruteforce)
    assert [(c["objective_c"], c["objective_q"]) for c in cands] == [(c["objective_c"], c["objective_q"]) for c in again]


def test_allocation_layer_table_has_the_stated_size():
    rows = si.unet_allocation_layers()
    total = sum(r[2] for r in rows)
    assert 2.5e9 < total < 2.6e9                      # the UNet the paper quantises has about 2.6 G parameters
    assert {r[1] for r in rows} == {"content", "quality"}
    assert sum(1 for r in rows if ".attn2.to_k" in r[0]) == 70     # 70 transformer blocks
    assert len({r[0] for r in rows}) == len(rows)
