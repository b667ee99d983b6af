"""Brute force over persistent schedules, through an operation-level simulator.

Independent of the recurrence: the simulator below knows only the operations of
the paper's Table 1 (what each consumes, produces, keeps and frees, its time and
its memory overhead); the enumerator knows only the *shape* of a persistent
schedule (Theorem, Section "Activation Checkpoint Solver / Modeling"): a segment
s..t either runs F_all^s, the schedule of s+1..t, B^s, or checkpoints its input,
runs F_ck^s, F_null^{s+1..s'-1}, then the schedule of s'..t, then the schedule of
s..s'-1.  Neither uses m_all / m_null or subtracts sizes from a budget.

Memory accounting of the simulator (the model behind the Theorem's thresholds):
  - every resident tensor counts with its size, except the segment's own input
    a^{s-1} (whoever owns the enclosing segment pays for it);
  - delta^t is resident from the start;
  - a forward operation peaks at resident + its output + o_f; F_null then frees
    its (plain) input;
  - B^j peaks at resident + o_b (its output delta^{j-1} is not counted while it
    runs), then frees delta^j, abar^j and a plain a^{j-1}; an abar^{j-1} stays.
"""
from __future__ import annotations

F_ALL, F_CK, F_NULL, BWD = 0, 1, 2, 3


def trees(s, t):
    """All decomposition trees of segment s..t."""
    if s == t:
        return [("leaf", s)]
    out = [("all", s, sub) for sub in trees(s + 1, t)]
    for sp in range(s + 1, t + 1):
        rights = trees(sp, t)
        lefts = trees(s, sp - 1)
        out += [("ck", s, sp, r, l) for r in rights for l in lefts]
    return out


def root_choice(tree):
    """Candidate number of the root decision: s for F_all (and leaves), s' for a checkpoint split."""
    return tree[2] if tree[0] == "ck" else tree[1]


def flatten(tree):
    kind = tree[0]
    if kind == "leaf":
        s = tree[1]
        return [(F_ALL, s), (BWD, s)]
    if kind == "all":
        _, s, sub = tree
        return [(F_ALL, s)] + flatten(sub) + [(BWD, s)]
    _, s, sp, right, left = tree
    return [(F_CK, s)] + [(F_NULL, j) for j in range(s + 1, sp)] + flatten(right) + flatten(left)


class ScheduleError(Exception):
    pass


def simulate(ops, s, t, uf, ub, wa, wabar, wdelta, of, ob, complete=True):
    """Run ops on segment s..t.  Returns (time, peak memory).  Stage arrays are
    indexed [k-1] for stage k; wa / wdelta are indexed 0..L.  With complete=False the
    list may be a prefix of a schedule: it need not end with the gradient of the input."""
    state = {("a", s - 1), ("delta", t)}

    def size(item):
        kind, j = item
        if kind == "a":
            return 0 if j == s - 1 else int(wa[j])
        if kind == "abar":
            return int(wabar[j - 1])
        return int(wdelta[j])

    def resident():
        return sum(size(i) for i in state)

    def has_a(j):
        return ("a", j) in state or ("abar", j) in state

    time = 0
    peak = 0
    for kind, j in ops:
        if kind in (F_ALL, F_CK, F_NULL):
            if not has_a(j - 1):
                raise ScheduleError(f"forward {j} without its input")
            if kind == F_NULL and ("a", j - 1) not in state:
                raise ScheduleError(f"F_null {j} needs a plain input")
            out = ("abar", j) if kind == F_ALL else ("a", j)
            if out in state:
                raise ScheduleError(f"{out} computed twice")
            peak = max(peak, resident() + size(out) + int(of[j - 1]))
            state.add(out)
            if kind == F_NULL:
                state.discard(("a", j - 1))
            time += int(uf[j - 1])
        else:
            if ("delta", j) not in state or ("abar", j) not in state or not has_a(j - 1):
                raise ScheduleError(f"backward {j} without its inputs")
            peak = max(peak, resident() + int(ob[j - 1]))
            state.discard(("delta", j))
            state.discard(("abar", j))
            state.discard(("a", j - 1))
            state.add(("delta", j - 1))
            time += int(ub[j - 1])
    if complete and ("delta", s - 1) not in state:
        raise ScheduleError("delta of the segment input was not produced")
    return time, peak


def brute_force_segment(s, t, M, uf, ub, wa, wabar, wdelta, of, ob, inf):
    """best[m], choice[m] for m = 0..M over every persistent schedule of s..t.
    choice is the smallest root candidate that attains the optimum, 0 if none fits."""
    per_choice = {}
    for tree in trees(s, t):
        time, peak = simulate(flatten(tree), s, t, uf, ub, wa, wabar, wdelta, of, ob)
        per_choice.setdefault(root_choice(tree), []).append((time, peak))
    best = [inf] * (M + 1)
    choice = [0] * (M + 1)
    for m in range(M + 1):
        for k in sorted(per_choice):
            fit = [tm for tm, pk in per_choice[k] if pk <= m]
            if fit and min(fit) < best[m]:
                best[m] = min(min(fit), inf)
                choice[m] = k
    return best, choice
