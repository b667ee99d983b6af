"""Pins of the CPU oracle against things other than itself.

Each test states what fixes the expected value: a hand-derived example, brute
force through the Table 1 simulator, a closed form, an invariant of the model.
"""
import os

import numpy as np
import pytest

from persistent_bruteforce import (BWD, F_ALL, F_CK, F_NULL, brute_force_segment, flatten, simulate, trees)
from workloads import make_config, random_chain_batch

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _load_worked_example():
    data = {"cost": {}, "choice": {}}
    with open(os.path.join(GOLDEN, "worked_example_L3.txt")) as fh:
        for line in fh:
            tok = line.split()
            if not tok or tok[0].startswith("#"):
                continue
            if tok[0] in ("uf", "ub", "wa", "wabar"):
                data[tok[0]] = [int(v) for v in tok[1:]]
            elif tok[0] == "M":
                data["M"] = int(tok[1])
            else:
                data[tok[0]][(int(tok[1]), int(tok[2]))] = tok[3:]
    return data


def test_worked_example(oracle_mod):
    g = _load_worked_example()
    cost, choice = oracle_mod.solve_chain(3, g["M"], g["uf"], g["ub"], g["wa"], g["wabar"])
    for (s, t), vals in g["cost"].items():
        want = [oracle_mod.INF if v == "X" else int(v) for v in vals]
        assert cost[s - 1, t - 1].tolist() == want, (s, t)
    for (s, t), vals in g["choice"].items():
        assert choice[s - 1, t - 1].tolist() == [int(v) for v in vals], (s, t)


def test_tree_counts():
    # number of persistent schedules of a chain of 1..6 stages (large Schroeder numbers)
    assert [len(trees(1, L)) for L in range(1, 7)] == [1, 2, 6, 22, 90, 394]


@pytest.mark.parametrize("L,seed,overheads,own_wd,zero", [
    (1, 10, False, False, False), (2, 11, True, True, False), (3, 12, False, False, False),
    (3, 13, True, False, False), (4, 14, True, True, False), (4, 15, False, True, True),
    (5, 16, True, True, False), (5, 17, False, False, False), (6, 18, True, True, False),
    (6, 19, False, False, True),
])
def test_brute_force_all_segments(oracle_mod, L, seed, overheads, own_wd, zero):
    """Every cell (s, t, m) and its recorded choice equal the optimum over all
    persistent schedules run through the operation simulator."""
    B = 6 if L <= 4 else 3
    size_hi = 5
    M = 3 * size_hi * 2 + 2 * size_hi * L  # past the point where nothing is infeasible
    batch = random_chain_batch(L, M, B, seed, size_hi=size_hi, overheads=overheads,
                               own_wdelta=own_wd, zero_sizes=zero)
    for b in range(B):
        ch = batch.chain(b)
        cost, choice = oracle_mod.solve_chain(L, M, *ch)
        for s in range(1, L + 1):
            for t in range(s, L + 1):
                best, pick = brute_force_segment(s, t, M, *ch, inf=oracle_mod.INF)
                assert cost[s - 1, t - 1].tolist() == best, (b, s, t)
                assert choice[s - 1, t - 1].tolist() == pick, (b, s, t)
        assert cost[0, L - 1, M] < oracle_mod.INF


@pytest.mark.parametrize("cfg", [0, 1])
def test_closed_form_unlimited_memory(oracle_mod, cfg):
    """With room for every abar the best schedule stores everything: cost is the sum of
    all forward and backward times and the choice is F_all (k = s)."""
    batch = make_config(cfg)
    uf, ub, wa, wabar, wd, of, ob = batch.chain(0)
    L = batch.L
    M = int(wd.max() + wabar.sum() + max(of.max(), ob.max())) + 3
    cost, choice = oracle_mod.solve_chain(L, M, uf, ub, wa, wabar, wd, of, ob)
    for s in range(1, L + 1):
        for t in range(s, L + 1):
            need = int(wd.max() + wabar[s - 1:t].sum() + max(of.max(), ob.max()))
            total = int(uf[s - 1:t].sum() + ub[s - 1:t].sum())
            assert (cost[s - 1, t - 1, need:] == total).all(), (s, t)
            assert (choice[s - 1, t - 1, need:] == s).all(), (s, t)


def _independent_min_memory(L, wa, wabar, wd, of, ob):
    """Smallest feasible budget of every segment by a scalar recursion over the same
    schedule shapes, written from the operation model rather than from the cost table:
    a leaf needs room for F_all then B; storing stage s adds abar^s under the rest;
    a checkpoint split needs the forward sweep, the right part above a^{s'-1}, the left part."""
    need = {}
    for d in range(L):
        for s in range(1, L - d + 1):
            t = s + d
            keep = max(wd[t] + wabar[s - 1] + of[s - 1], wd[s] + wabar[s - 1] + ob[s - 1])
            if d == 0:
                need[s, t] = keep
                continue
            opt_all = max(keep, wabar[s - 1] + need[s + 1, t])
            sweep = wd[t] + max([wa[s] + of[s - 1]] +
                                [wa[j - 1] + wa[j] + of[j - 1] for j in range(s + 1, t)])
            opt_ck = max(sweep, min(max(wa[sp - 1] + need[sp, t], need[s, sp - 1])
                                    for sp in range(s + 1, t + 1)))
            need[s, t] = min(opt_all, opt_ck)
    return need


@pytest.mark.parametrize("which", ["cfg0", "cfg1", "rand_ovh", "rand_zero"])
def test_invariants_and_first_feasible_column(oracle_mod, which):
    if which == "cfg0":
        batch = make_config(0)
    elif which == "cfg1":
        batch = make_config(1)
    elif which == "rand_ovh":
        batch = random_chain_batch(12, 90, 1, 77, size_hi=7, overheads=True, own_wdelta=True)
    else:
        batch = random_chain_batch(10, 60, 1, 78, size_hi=5, zero_sizes=True)
    L, M = batch.L, batch.M
    uf, ub, wa, wabar, wd, of, ob = (a.astype(np.int64) for a in batch.chain(0))
    cost, choice = oracle_mod.solve_chain(L, M, *batch.chain(0))
    INF = oracle_mod.INF
    need = _independent_min_memory(L, wa, wabar, wd, of, ob)
    for s in range(1, L + 1):
        for t in range(s, L + 1):
            row = cost[s - 1, t - 1].astype(np.int64)
            pick = choice[s - 1, t - 1]
            # more memory never hurts
            assert (np.diff(row) <= 0).all(), (s, t)
            # no schedule beats running every forward and backward once
            lower = int(uf[s - 1:t].sum() + ub[s - 1:t].sum())
            assert (row[row < INF] >= lower).all(), (s, t)
            # every stage must run B^k with delta^k and abar^k resident
            floor = max(int(wd[k] + wabar[k - 1] + ob[k - 1]) for k in range(s, t + 1))
            assert (row[:min(floor, M + 1)] == INF).all(), (s, t)
            # choice 0 <=> infeasible, otherwise a candidate of this cell
            assert ((pick == 0) == (row == INF)).all(), (s, t)
            assert ((pick[row < INF] >= s) & (pick[row < INF] <= t)).all(), (s, t)
            # first feasible column = independent minimum-memory recursion
            first = int(np.argmax(row < INF)) if (row < INF).any() else M + 1
            assert first == min(need[s, t], M + 1), (s, t, first, need[s, t])


def test_single_stage(oracle_mod):
    # L = 1: u_f + u_b once delta^1, abar^1 and the larger overhead fit
    cost, choice = oracle_mod.solve_chain(1, 20, [7], [9], [2, 3], [5], [4, 6], [2], [1])
    need = 6 + 5 + 2
    assert (cost[0, 0, :need] == oracle_mod.INF).all() and (cost[0, 0, need:] == 16).all()
    assert (choice[0, 0, :need] == 0).all() and (choice[0, 0, need:] == 1).all()


def test_thresholds_match_simulated_peaks(oracle_mod):
    """m_all^{s,s} is the simulated peak of F_all^s, B^s; m_null^{s,t} is the simulated peak of
    the forward sweep F_ck^s, F_null^{s+1..t-1} run as a prefix of a schedule of s..t (delta^t
    resident, segment input free) through the set-based simulator, which knows only Table 1."""
    for seed, ovh, wd_own in [(5, True, True), (6, False, False), (7, True, False), (8, False, True)]:
        batch = random_chain_batch(7, 10, 2, seed, size_hi=9, overheads=ovh, own_wdelta=wd_own)
        for b in range(batch.B):
            uf, ub, wa, wabar, wd, of, ob = batch.chain(b)
            L = batch.L
            for s in range(1, L + 1):
                m_all, _ = oracle_mod.thresholds(L, wa, wabar, wd, of, ob, s, s)
                _, peak = simulate([(F_ALL, s), (BWD, s)], s, s, uf, ub, wa, wabar, wd, of, ob)
                assert m_all == peak
                for t in range(s + 1, L + 1):
                    _, m_null = oracle_mod.thresholds(L, wa, wabar, wd, of, ob, s, t)
                    sweep = [(F_CK, s)] + [(F_NULL, j) for j in range(s + 1, t)]
                    _, peak = simulate(sweep, s, t, uf, ub, wa, wabar, wd, of, ob, complete=False)
                    assert m_null == peak, (s, t)


@pytest.mark.parametrize("cfg", [0, 1])
def test_reconstructed_schedule_runs_in_budget(oracle_mod, cfg):
    """The operation list rebuilt from the recorded choices takes exactly the table's
    time and fits the budget when run through the simulator."""
    batch = make_config(cfg)
    ch = batch.chain(0)
    L, M = batch.L, batch.M
    cost, choice = oracle_mod.solve_chain(L, M, *ch)
    checked = 0
    for m in range(0, M + 1, max(1, M // 40)):
        if cost[0, L - 1, m] >= oracle_mod.INF:
            continue
        ops = oracle_mod.reconstruct(choice, ch[2], ch[3], 1, L, m)
        time, peak = simulate(ops, 1, L, *ch)
        assert time == cost[0, L - 1, m] and peak <= m
        checked += 1
    assert checked > 3
    with pytest.raises(ValueError):
        oracle_mod.reconstruct(choice, ch[2], ch[3], 1, L, 0)


def test_threads_do_not_change_results(oracle_mod):
    batch = make_config(1)
    a = oracle_mod.solve_chain(batch.L, batch.M, *batch.chain(0), nthreads=1)
    b = oracle_mod.solve_chain(batch.L, batch.M, *batch.chain(0), nthreads=4)
    assert (a[0] == b[0]).all() and (a[1] == b[1]).all()
