"""Pins of the oracle's planner-side steps: plan selection and bytes-to-slots discretisation."""
import random

import numpy as np
import pytest

from workloads import make_config


def test_discretize_is_the_least_slot_count_that_covers_the_size(oracle_mod):
    """ceil(size*M/budget) is characterised by: slots*budget >= size*M > (slots-1)*budget."""
    rng = random.Random(3)
    for _ in range(300):
        M = rng.choice([1, 7, 64, 4096, 1 << 20])
        budget = rng.randrange(1, 1 << 40)
        sizes = [0, 1, budget, budget - 1, budget + 1] + [rng.randrange(0, 1 << 41) for _ in range(6)]
        for v, s in zip(sizes, oracle_mod.discretize(sizes, budget, M)):
            if s == oracle_mod.SLOT_MAX:
                assert v * M > (s - 1) * budget
                continue
            assert s * budget >= v * M and (s == 0 or (s - 1) * budget < v * M), (v, M, budget, s)


def test_discretize_special_cases(oracle_mod):
    assert oracle_mod.discretize([0, 10, 20, 25], 100, 10) == [0, 1, 2, 3]       # exact multiples stay, 2.5 -> 3
    assert oracle_mod.discretize([100], 100, 64) == [64]                          # the whole budget is M slots
    assert oracle_mod.discretize([1], 1 << 40, 4096) == [1]                       # anything nonzero takes a slot
    assert oracle_mod.discretize([1 << 41], 1, 1 << 20) == [oracle_mod.SLOT_MAX]  # clamp
    with pytest.raises(ValueError):
        oracle_mod.discretize([1], 0, 8)


def test_discretize_is_conservative_for_schedules(oracle_mod):
    """A set of tensors that fits in slots fits in bytes: sum(slots) <= M  =>  sum(bytes) <= budget."""
    rng = random.Random(4)
    for _ in range(200):
        M = rng.choice([16, 100, 1024])
        budget = rng.randrange(1000, 1 << 30)
        sizes = [rng.randrange(0, budget // 3) for _ in range(rng.randrange(1, 6))]
        slots = oracle_mod.discretize(sizes, budget, M)
        if sum(slots) <= M:
            assert sum(sizes) <= budget


def test_select_plan_cases(oracle_mod):
    batch = make_config(2)
    L, M = batch.L, batch.M
    tables = [oracle_mod.solve_chain(L, M, *batch.chain(b))[0] for b in range(4)]
    roots = [int(t[0, L - 1, M]) for t in tables]
    b, v = oracle_mod.select_plan(tables, L, [M] * 4)
    assert v == min(roots) and b == roots.index(min(roots))
    # a tie goes to the smaller index
    b2, _ = oracle_mod.select_plan([tables[1], tables[1], tables[0]], L, [M, M, 0])
    assert b2 == 0
    # budgets below the frontier are infeasible; none feasible -> (-1, INF)
    assert oracle_mod.select_plan(tables, L, [0, -5, 1, 2]) == (-1, oracle_mod.INF)
    # a budget above M reads column M
    assert oracle_mod.select_plan(tables[:1], L, [M + 1000]) == (0, roots[0])
    # the choice depends on the per-chain budget: starve the winner
    need = next(m for m in range(M + 1) if tables[b][0, L - 1, m] < oracle_mod.INF)
    budgets = [M] * 4
    budgets[b] = need - 1
    b3, v3 = oracle_mod.select_plan(tables, L, budgets)
    assert b3 != b and v3 == min(r for k, r in enumerate(roots) if k != b)


def test_budget_sweep_closed_forms_and_bracket(oracle_mod):
    from fractions import Fraction
    assert oracle_mod.budget_sweep(1000, 0, 1, 5) == [1000] * 5                       # alpha = 0
    assert oracle_mod.budget_sweep(3, 1, 1, 6) == [3, 6, 12, 24, 48, 96]              # alpha = 1 doubles
    assert oracle_mod.budget_sweep(1000, 1, 10, 4) == [1000, 1100, 1210, 1331]        # 1.1^n, exact
    assert oracle_mod.budget_sweep(7, 1, 2, 4) == [7, 10, 15, 23]                     # 7 * 1.5^n = 7, 10.5, 15.75, 23.625
    for base, num, den in ((80 * 2**30, 1, 10), (12345678901, 3, 20), (1, 1, 8), (999, 7, 100)):
        got = oracle_mod.budget_sweep(base, num, den, 10)
        for n, b in enumerate(got):
            exact = base * (1 + Fraction(num, den)) ** n
            assert b <= exact < b + 1
        assert got == sorted(got) and got[0] == base
    for bad in ((0, 1, 10, 3), (5, -1, 10, 3), (5, 1, 0, 3), (5, 1, 10, 0)):
        with pytest.raises(ValueError):
            oracle_mod.budget_sweep(*bad)


def test_discretize_sweep_rows_are_single_discretisations(oracle_mod):
    sizes = [0, 1, 999, 1000, 1001, 123456]
    rows = oracle_mod.discretize_sweep(sizes, 1000, 1, 10, 4, 100)
    assert rows[0] == [0, 1, 100, 100, 101, 12346]          # budget 1000: ceil(v / 10)
    assert rows[1] == [0, 1, 91, 91, 91, 11224]             # budget 1100: ceil(v * 100 / 1100)
    for row, budget in zip(rows, (1000, 1100, 1210, 1331)):
        assert row == oracle_mod.discretize(sizes, budget, 100)
    # a larger budget never needs more slots
    assert all(a >= b for r0, r1 in zip(rows, rows[1:]) for a, b in zip(r0, r1))
