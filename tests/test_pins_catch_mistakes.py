"""The pins are only worth something if a plausible mistake trips them.

A small pure-Python evaluation of the Theorem (Section "Activation Checkpoint
Solver / Modeling") serves twice: unmodified it is a second opinion on the C
oracle; with one planted mistake at a time (on the CPU, in this file only) it
must disagree with the brute force over persistent schedules.
"""
import numpy as np
import pytest

from persistent_bruteforce import F_CK, F_NULL, brute_force_segment, simulate
from workloads import make_config, random_chain_batch

INF = 1 << 30


def py_table(L, M, uf, ub, wa, wabar, wd, of, ob, mistake=None):
    C = {}
    K = {}

    def get(s, t, m):
        return INF if m < 0 else C[s, t][m]

    for d in range(L):
        for s in range(1, L - d + 1):
            t = s + d
            m_all = max(wd[t] + wabar[s - 1] + of[s - 1], wd[s] + wabar[s - 1] + ob[s - 1])
            if mistake == "m_all_without_backward_term":
                m_all = wd[t] + wabar[s - 1] + of[s - 1]
            if mistake == "m_all_uses_a_not_abar":
                m_all = max(wd[t] + wa[s] + of[s - 1], wd[s] + wa[s] + ob[s - 1])
            m_null = wd[t] + max([wa[s] + of[s - 1]] +
                                 [wa[j - 1] + wa[j] + of[j - 1] for j in range(s + 1, t)])
            if mistake == "no_m_null_gate":
                m_null = 0
            cost = [INF] * (M + 1)
            pick = [0] * (M + 1)
            for m in range(M + 1):
                best, arg = INF, 0
                if m >= m_all:
                    if d == 0:
                        v = uf[s - 1] + ub[s - 1]
                    else:
                        shift = wabar[s - 1]
                        if mistake == "all_shift_uses_a":
                            shift = wa[s]
                        v = uf[s - 1] + ub[s - 1] + get(s + 1, t, m - shift)
                        if mistake == "all_drops_backward_time":
                            v -= ub[s - 1]
                    v = min(v, INF)
                    if v < best:
                        best, arg = v, s
                if d > 0 and m >= m_null:
                    for sp in range(s + 1, t + 1):
                        fwd = sum(uf[s - 1:sp - 1])
                        if mistake == "ck_drops_forward_sum":
                            fwd = 0
                        if mistake == "ck_forward_sum_one_short":
                            fwd = sum(uf[s - 1:sp - 2])
                        shift = wa[sp - 1]
                        if mistake == "ck_shift_index_off_by_one":
                            shift = wa[sp]
                        right = get(sp, t, m - shift)
                        left = get(s, sp - 1, m)
                        if mistake == "ck_shift_on_wrong_operand":
                            right, left = get(sp, t, m), get(s, sp - 1, m - shift)
                        if mistake == "ck_no_shift":
                            right = get(sp, t, m)
                        v = min(fwd + right + left, INF)
                        if v < best or (mistake == "ties_to_largest" and v == best and v < INF):
                            best, arg = v, sp
                cost[m], pick[m] = best, arg
            C[s, t], K[s, t] = cost, pick
    return C, K


MISTAKES = ["m_all_without_backward_term", "m_all_uses_a_not_abar", "all_shift_uses_a",
            "all_drops_backward_time", "ck_drops_forward_sum", "ck_forward_sum_one_short",
            "ck_shift_index_off_by_one", "ck_shift_on_wrong_operand", "ck_no_shift", "ties_to_largest"]


def _cases():
    out = []
    for L, seed in [(3, 101), (4, 102), (5, 103), (5, 104)]:
        batch = random_chain_batch(L, 14 * L, 4, seed, size_hi=6, overheads=True, own_wdelta=True)
        out += [(batch.L, batch.M, [a.tolist() for a in batch.chain(b)]) for b in range(batch.B)]
    return out


def _disagrees_with_brute_force(mistake):
    for L, M, ch in _cases():
        C, K = py_table(L, M, *ch, mistake=mistake)
        for s in range(1, L + 1):
            for t in range(s, L + 1):
                best, pick = brute_force_segment(s, t, M, *ch, inf=INF)
                if C[s, t] != best or K[s, t] != pick:
                    return True
    return False


def test_unmodified_python_table_passes_brute_force():
    assert not _disagrees_with_brute_force(None)


@pytest.mark.parametrize("mistake", MISTAKES)
def test_planted_mistake_is_caught(mistake):
    assert _disagrees_with_brute_force(mistake), mistake


def test_m_null_gate_is_implied_when_abar_contains_a():
    """With omega_abar >= omega_a the m_null gate never changes a cell: every forward of the
    sweep is run again, with at least the same residents, inside the recursive parts.  So the
    brute force cannot pin it; it is pinned by test_thresholds_match_simulated_peaks."""
    for L, M, ch in _cases():
        assert py_table(L, M, *ch, mistake="no_m_null_gate") == py_table(L, M, *ch)


def _m_null(wa, wd, of, s, t, mistake=None):
    """The Theorem's m_null^{s,t}, with one planted mistake at a time."""
    lo, hi = s + 1, t                    # inner maximum over lo <= j < hi
    if mistake == "sweep_stops_one_stage_early":
        hi = t - 1
    if mistake == "sweep_includes_stage_t":
        hi = t + 1
    first = wa[s] + of[s - 1]
    if mistake == "first_forward_without_overhead":
        first = wa[s]
    inner = [wa[j - 1] + wa[j] + of[j - 1] for j in range(lo, min(hi, len(wa)))]
    if mistake == "input_of_f_null_not_counted":
        inner = [wa[j] + of[j - 1] for j in range(lo, hi)]
    if mistake == "overhead_of_the_wrong_stage":
        inner = [wa[j - 1] + wa[j] + of[j - 2] for j in range(lo, hi)]
    total = wd[t] + max([first] + inner)
    if mistake == "delta_of_the_segment_end_forgotten":
        total -= wd[t]
    if mistake == "delta_of_the_wrong_end":
        total += wd[s - 1] - wd[t]
    return total


M_NULL_MISTAKES = ["sweep_stops_one_stage_early", "sweep_includes_stage_t", "first_forward_without_overhead",
                   "input_of_f_null_not_counted", "overhead_of_the_wrong_stage",
                   "delta_of_the_segment_end_forgotten", "delta_of_the_wrong_end"]


def _m_null_disagrees_with_simulated_sweep(mistake):
    """m_null is not visible to the brute force (see the test above); its pin is the peak of the
    forward sweep F_ck^s, F_null^{s+1..t-1} in the set-based simulator, delta^t resident."""
    for L, _, ch in _cases():
        uf, ub, wa, wabar, wd, of, ob = ch
        for s in range(1, L + 1):
            for t in range(s + 1, L + 1):
                sweep = [(F_CK, s)] + [(F_NULL, j) for j in range(s + 1, t)]
                _, peak = simulate(sweep, s, t, uf, ub, wa, wabar, wd, of, ob, complete=False)
                if _m_null(wa, wd, of, s, t, mistake) != peak:
                    return True
    return False


def test_unmodified_m_null_matches_the_simulated_sweep():
    assert not _m_null_disagrees_with_simulated_sweep(None)


@pytest.mark.parametrize("mistake", M_NULL_MISTAKES)
def test_planted_m_null_mistake_is_caught(mistake):
    assert _m_null_disagrees_with_simulated_sweep(mistake), mistake


@pytest.mark.parametrize("cfg", [0, 1])
def test_second_opinion_on_c_oracle(oracle_mod, cfg):
    batch = make_config(cfg)
    L, M = batch.L, (batch.M if cfg == 0 else 96)
    ch = batch.chain(0)
    cost, choice = oracle_mod.solve_chain(L, M, *ch)
    C, K = py_table(L, M, *[a.tolist() for a in ch])
    for (s, t), row in C.items():
        assert cost[s - 1, t - 1].tolist() == row, (s, t)
        assert choice[s - 1, t - 1].tolist() == K[s, t], (s, t)


def test_second_opinion_when_abar_smaller_than_a(oracle_mod):
    """Inputs that break omega_abar >= omega_a are outside the Theorem's model; the C oracle and
    the Python evaluation still agree on what the printed formulas give (formula conformance,
    not parity with an optimum)."""
    rng = np.random.default_rng(9)
    L, M = 9, 60
    uf = rng.integers(1, 50, L); ub = rng.integers(1, 90, L)
    wa = rng.integers(1, 9, L + 1); wabar = rng.integers(0, 6, L)
    wd = rng.integers(0, 7, L + 1); of = rng.integers(0, 4, L); ob = rng.integers(0, 4, L)
    cost, choice = oracle_mod.solve_chain(L, M, uf, ub, wa, wabar, wd, of, ob)
    C, K = py_table(L, M, *[a.tolist() for a in (uf, ub, wa, wabar, wd, of, ob)])
    for (s, t), row in C.items():
        assert cost[s - 1, t - 1].tolist() == row and choice[s - 1, t - 1].tolist() == K[s, t]


def test_the_theorem_needs_abar_to_contain_a(oracle_mod):
    """Why omega_abar >= omega_a is a precondition of the library: without it the recurrence is
    not the optimum over persistent schedules any more (the brute force finds cheaper or
    earlier-fitting schedules), so such inputs have no exact answer to be compared with."""
    rng = np.random.default_rng(5)
    differs = 0
    for _ in range(25):
        L, M = int(rng.integers(3, 6)), 40
        uf = rng.integers(1, 50, L); ub = rng.integers(1, 90, L)
        wa = rng.integers(1, 9, L + 1); wabar = rng.integers(0, 6, L)
        wd = rng.integers(0, 7, L + 1); of = rng.integers(0, 4, L); ob = rng.integers(0, 4, L)
        cost, _ = oracle_mod.solve_chain(L, M, uf, ub, wa, wabar, wd, of, ob)
        best, _ = brute_force_segment(1, L, M, uf, ub, wa, wabar, wd, of, ob, INF)
        differs += cost[0, L - 1].tolist() != best
    assert differs > 0
