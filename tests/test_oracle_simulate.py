"""Pins of the oracle's operation-list simulator (oracle.simulate).

It is checked against figures derived by hand from Table 1 ("List of Operations") for the
3-stage worked example, against the independent simulator of tests/persistent_bruteforce.py
(written separately, state kept as a set of tensors) on every persistent schedule of short
chains and on random, mostly invalid, lists, and against the table of the recurrence.
"""
import os

import numpy as np
import pytest

import persistent_bruteforce as bf
from workloads.chains import random_chain_batch

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
KIND = {"A": 0, "C": 1, "N": 2, "B": 3}


def load_schedules():
    chain, rows = {}, []
    with open(os.path.join(GOLDEN, "worked_example_L3.txt")) as f:
        for line in f:
            tok = line.split()
            if tok and tok[0] in ("uf", "ub", "wa", "wabar"):
                chain[tok[0]] = [int(v) for v in tok[1:]]
    with open(os.path.join(GOLDEN, "worked_example_L3_schedules.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            m, ops, time, peak = [p.strip() for p in line.split("|")]
            rows.append((int(m), [(KIND[o[0]], int(o[1:])) for o in ops.split()], int(time), int(peak)))
    return chain, rows


def test_hand_executed_schedules(oracle_mod):
    chain, rows = load_schedules()
    assert len(rows) == 5
    cost, choice = oracle_mod.solve_chain(3, 16, chain["uf"], chain["ub"], chain["wa"], chain["wabar"])
    for m, ops, time, peak in rows:
        assert oracle_mod.simulate(ops, 3, chain["uf"], chain["ub"], chain["wa"], chain["wabar"]) == (time, peak)
        # the list is the one the recorded choices give at that budget, and it first fits at its peak
        assert oracle_mod.reconstruct(choice, chain["wa"], chain["wabar"], 1, 3, m) == ops
        assert cost[0, 2, m] == time and peak <= m


@pytest.mark.parametrize("L", [1, 2, 3, 4, 5])
def test_every_persistent_schedule_matches_the_set_based_simulator(oracle_mod, L):
    batch = random_chain_batch(L, 8, 3, 70 + L, size_hi=5, time_hi=50, overheads=True, own_wdelta=True)
    for b in range(batch.B):
        uf, ub, wa, wabar, wd, of, ob = batch.chain(b)
        for tree in bf.trees(1, L):
            ops = bf.flatten(tree)
            assert oracle_mod.simulate(ops, L, uf, ub, wa, wabar, wd, of, ob) == \
                bf.simulate(ops, 1, L, uf, ub, wa, wabar, wd, of, ob)


def test_mutated_lists_agree_on_validity_and_value(oracle_mod):
    """Persistent schedules with one or two random edits (an operation dropped, repeated, moved,
    or its kind or stage changed): mostly invalid, sometimes still executable."""
    rng = np.random.default_rng(5)
    L = 4
    batch = random_chain_batch(L, 8, 1, 77, size_hi=6, time_hi=40, overheads=True, own_wdelta=True)
    uf, ub, wa, wabar, wd, of, ob = batch.chain(0)
    base = [bf.flatten(t) for t in bf.trees(1, L)]
    valid = invalid = 0
    for _ in range(4000):
        ops = list(base[int(rng.integers(len(base)))])
        for _ in range(int(rng.integers(1, 3))):
            i = int(rng.integers(len(ops)))
            edit = int(rng.integers(5))
            if edit == 0:
                del ops[i]
            elif edit == 1:
                ops.insert(i, ops[i])
            elif edit == 2:
                ops.insert(int(rng.integers(len(ops))), ops.pop(i))
            elif edit == 3:
                ops[i] = (int(rng.integers(0, 4)), ops[i][1])
            else:
                ops[i] = (ops[i][0], int(rng.integers(1, L + 1)))
            if not ops:
                break
        try:
            want = bf.simulate(ops, 1, L, uf, ub, wa, wabar, wd, of, ob)
        except bf.ScheduleError:
            want = None
        try:
            got = oracle_mod.simulate(ops, L, uf, ub, wa, wabar, wd, of, ob)
        except ValueError:
            got = None
        assert got == want, ops
        valid += want is not None
        invalid += want is None
    assert valid > 50 and invalid > 50  # the sweep reaches both kinds


def test_rejects_malformed_lists(oracle_mod):
    args = (2, [1, 1], [1, 1], [1, 1, 1], [1, 1])
    for ops in ([(0, 0), (3, 1)], [(0, 3)], [(4, 1)], [(3, 1)], [(0, 1)], [(0, 1), (0, 1)], []):
        with pytest.raises(ValueError):
            oracle_mod.simulate(ops, *args)


@pytest.mark.parametrize("seed", range(4))
def test_table_cost_is_the_simulated_time_and_the_budget_holds(oracle_mod, seed):
    L, M = 7, 60
    batch = random_chain_batch(L, M, 1, 300 + seed, size_hi=6, time_hi=500, overheads=bool(seed & 1),
                               own_wdelta=bool(seed & 2))
    uf, ub, wa, wabar, wd, of, ob = batch.chain(0)
    cost, choice = oracle_mod.solve_chain(L, M, uf, ub, wa, wabar, wd, of, ob)
    seen = 0
    for m in range(M + 1):
        if cost[0, L - 1, m] >= oracle_mod.INF:
            continue
        time, peak = oracle_mod.simulate(oracle_mod.reconstruct(choice, wa, wabar, 1, L, m), L, uf, ub, wa, wabar,
                                         wd, of, ob)
        assert time == cost[0, L - 1, m] and peak <= m
        # the schedule is optimal for its own peak too
        assert cost[0, L - 1, peak] == time
        seen += 1
    assert seen > 0
