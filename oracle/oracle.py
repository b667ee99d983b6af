"""ctypes front end of the CPU oracle (oracle/ckpt_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  Nothing in the GPU package imports this module
and this module imports nothing from the GPU package.

solve_chain / solve_batch evaluate the recurrence of the paper's Theorem
(Section "Activation Checkpoint Solver / Modeling"); reconstruct() walks the
recorded choices into the operation sequence of Table 1; simulate() executes such
a sequence under the memory model of Table 1.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

INF = 1 << 30
_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ckpt_oracle.c")
_LIB = os.path.join(_HERE, "libckpt_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
                               "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        p32 = ctypes.POINTER(ctypes.c_int32)
        lib.oracle_solve_chain.restype = ctypes.c_int
        lib.oracle_solve_chain.argtypes = [ctypes.c_int, ctypes.c_int] + [p32] * 7 + [
            p32, ctypes.POINTER(ctypes.c_int16), ctypes.c_int]
        for f in (lib.oracle_m_all, lib.oracle_m_null):
            f.restype = ctypes.c_int64
            f.argtypes = [ctypes.c_int] + [p32] * 5 + [ctypes.c_int, ctypes.c_int]
        lib.oracle_max_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _p(a, ct=ctypes.c_int32):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a


def max_threads() -> int:
    return _load().oracle_max_threads()


def solve_chain(L, M, uf, ub, wa, wabar, wdelta=None, of=None, ob=None, nthreads=1):
    """One chain -> (cost int32 [L, L, M+1], choice int16 [L, L, M+1]).

    Index [s-1, t-1, m]; entries with s > t are cost 0 / choice -1 (never written).
    """
    uf, ub, wa, wabar = map(_i32, (uf, ub, wa, wabar))
    wd = wa if wdelta is None else _i32(wdelta)
    of = np.zeros(L, np.int32) if of is None else _i32(of)
    ob = np.zeros(L, np.int32) if ob is None else _i32(ob)
    assert uf.shape == (L,) and ub.shape == (L,) and wabar.shape == (L,)
    assert wa.shape == (L + 1,) and wd.shape == (L + 1,) and of.shape == (L,) and ob.shape == (L,)
    cost = np.zeros((L, L, M + 1), np.int32)
    choice = np.full((L, L, M + 1), -1, np.int16)
    rc = _load().oracle_solve_chain(L, M, _p(uf), _p(ub), _p(wa), _p(wabar), _p(wd), _p(of), _p(ob),
                                    _p(cost), _p(choice, ctypes.c_int16), int(nthreads))
    if rc != 0:
        raise ValueError("oracle_solve_chain: bad argument")
    return cost, choice


def solve_batch(batch, nthreads=1):
    """workloads.ChainBatch -> list of (cost, choice) per chain."""
    return [solve_chain(batch.L, batch.M, *batch.chain(b), nthreads=nthreads) for b in range(batch.B)]


def thresholds(L, wa, wabar, wdelta, of, ob, s, t):
    """(m_all^{s,t}, m_null^{s,t}) of the Theorem's last display."""
    wa, wabar, wdelta, of, ob = map(_i32, (wa, wabar, wdelta, of, ob))
    lib = _load()
    args = (L, _p(wa), _p(wabar), _p(wdelta), _p(of), _p(ob), s, t)
    return int(lib.oracle_m_all(*args)), int(lib.oracle_m_null(*args))


# Operation kinds of Table 1.
F_ALL, F_CK, F_NULL, BWD = 0, 1, 2, 3


def reconstruct(choice, wa, wabar, s, t, m):
    """Operation list [(kind, stage), ...] that realises C_BP(s, t, m).

    Follows the recorded choice k of each visited cell: k == s with s == t is
    F_all^s, B^s; k == s is F_all^s, the schedule of (s+1, t, m - omega_abar^s),
    B^s (C_all of the Theorem); k = s' > s is F_ck^s, F_null^{s+1..s'-1}, the
    schedule of (s', t, m - omega_a^{s'-1}), the schedule of (s, s'-1, m) (C_ck).
    Raises ValueError on an infeasible cell.
    """
    if m < 0:
        raise ValueError("infeasible")
    k = int(choice[s - 1, t - 1, m])
    if k == 0:
        raise ValueError("infeasible")
    if s == t:
        return [(F_ALL, s), (BWD, s)]
    if k == s:
        return ([(F_ALL, s)] + reconstruct(choice, wa, wabar, s + 1, t, m - int(wabar[s - 1]))
                + [(BWD, s)])
    ops = [(F_CK, s)] + [(F_NULL, j) for j in range(s + 1, k)]
    ops += reconstruct(choice, wa, wabar, k, t, m - int(wa[k - 1]))
    ops += reconstruct(choice, wa, wabar, s, k - 1, m)
    return ops


def block_indices(ops, L):
    """Activation-checkpoint block index of every stage (Section "Code generation": each node is
    annotated with the index of its checkpoint block, nodes with the same index are packaged
    into one function that is wrapped in the framework's checkpoint call, which keeps the
    block's input and recomputes its inside during the backward phase).

    Read off an operation list of Table 1 over stages 1..L.  A stage's annotation comes from the
    FIRST forward operation it receives (its later forwards are the recomputation itself):
      F_all^j   keeps abar^j: stage j lies in no checkpoint block, index -1;
      F_ck^j    keeps only the input a^{j-1} and the output a^j: stage j opens a new block;
      F_null^j  keeps nothing of its own: stage j continues the block of stage j-1.
    Blocks are numbered 0, 1, ... in chain order.  Returns (list of L indices, number of blocks).
    Raises ValueError if some stage has no forward operation, or if a first F_null^j does not
    follow a stage that is inside a block.
    """
    first = {}
    for kind, j in ops:
        kind, j = int(kind), int(j)
        if kind in (F_ALL, F_CK, F_NULL) and j not in first:
            first[j] = kind
    block, nblocks = [], 0
    for j in range(1, L + 1):
        if j not in first:
            raise ValueError(f"stage {j} is never run forward")
        if first[j] == F_ALL:
            block.append(-1)
        elif first[j] == F_CK:
            block.append(nblocks)
            nblocks += 1
        else:
            if j == 1 or block[-1] < 0:
                raise ValueError(f"F_null^{j} does not continue a checkpoint block")
            block.append(block[-1])
    return block, nblocks


def simulate(ops, L, uf, ub, wa, wabar, wdelta=None, of=None, ob=None):
    """Run an operation list over the whole chain 1..L and return (time, peak memory).

    The operations are those of Table 1 ("List of Operations"): F_all^j and F_ck^j read
    a^{j-1} (plain, or inside abar^{j-1}), keep it and add abar^j resp. a^j; F_null^j reads a
    plain a^{j-1}, adds a^j and drops a^{j-1}; B^j reads delta^j, abar^j and a^{j-1} (plain or
    inside abar^{j-1}), adds delta^{j-1} and drops delta^j, abar^j and a plain a^{j-1}.  An
    operation takes u_f^j resp. u_b^j and needs o_f^j resp. o_b^j on top of what is resident.

    Memory is counted the way the Theorem's thresholds count it: the chain input a^0 is free,
    delta^L is resident from the start, a forward operation needs room for its output while it
    runs, B^j does not count its output delta^{j-1} while it runs.
    Raises ValueError for a list that cannot be executed (a missing operand, a tensor computed
    while it is still resident, an unknown operation) or that ends without delta^0.
    """
    wd = wa if wdelta is None else wdelta
    of = [0] * L if of is None else of
    ob = [0] * L if ob is None else ob
    plain = [False] * (L + 1)   # a^j resident on its own
    full = [False] * (L + 1)    # abar^j resident (contains a^j)
    grad = [False] * (L + 1)    # delta^j resident
    plain[0] = True
    grad[L] = True

    def resident():
        total = 0
        for j in range(L + 1):
            if plain[j] and j > 0:
                total += int(wa[j])
            if full[j]:
                total += int(wabar[j - 1])
            if grad[j]:
                total += int(wd[j])
        return total

    time = peak = 0
    for kind, j in ops:
        kind, j = int(kind), int(j)
        if not 1 <= j <= L:
            raise ValueError(f"stage {j} outside the chain")
        if kind in (F_ALL, F_CK, F_NULL):
            if not (plain[j - 1] or full[j - 1]):
                raise ValueError(f"forward of stage {j} without a^{j - 1}")
            if kind == F_NULL and not plain[j - 1]:
                raise ValueError(f"F_null^{j} needs a plain a^{j - 1}")
            made = full if kind == F_ALL else plain
            if made[j]:
                raise ValueError(f"output of stage {j} is already resident")
            size = int(wabar[j - 1]) if kind == F_ALL else int(wa[j])
            peak = max(peak, resident() + size + int(of[j - 1]))
            made[j] = True
            if kind == F_NULL:
                plain[j - 1] = False
            time += int(uf[j - 1])
        elif kind == BWD:
            if not (grad[j] and full[j] and (plain[j - 1] or full[j - 1])):
                raise ValueError(f"B^{j} without its operands")
            peak = max(peak, resident() + int(ob[j - 1]))
            grad[j] = full[j] = plain[j - 1] = False
            grad[j - 1] = True
            time += int(ub[j - 1])
        else:
            raise ValueError(f"unknown operation {kind}")
    if not grad[0]:
        raise ValueError("the list ends without delta^0")
    return time, peak


def min_feasible_memory(L, wa, wabar, wdelta=None, of=None, ob=None):
    """need[s-1, t-1] = smallest m with C_BP(s, t, m) finite (int64 [L, L], s <= t).

    Scalar form of the Theorem's feasibility: a leaf needs m_all^{s,s}; storing stage s
    needs max(m_all^{s,t}, omega_abar^s + need(s+1, t)); a checkpoint split at s' needs
    max(m_null^{s,t}, omega_a^{s'-1} + need(s', t), need(s, s'-1)).
    """
    wa = np.asarray(wa, np.int64)
    wabar = np.asarray(wabar, np.int64)
    wd = wa if wdelta is None else np.asarray(wdelta, np.int64)
    of = np.zeros(L, np.int64) if of is None else np.asarray(of, np.int64)
    ob = np.zeros(L, np.int64) if ob is None else np.asarray(ob, np.int64)
    need = np.zeros((L + 2, L + 2), np.int64)  # 1-based
    for s in range(1, L + 1):
        need[s, s] = max(wd[s] + wabar[s - 1] + of[s - 1], wd[s] + wabar[s - 1] + ob[s - 1])
    for d in range(1, L):
        for s in range(1, L - d + 1):
            t = s + d
            m_all = max(wd[t] + wabar[s - 1] + of[s - 1], wd[s] + wabar[s - 1] + ob[s - 1])
            sweep = wa[s] + of[s - 1]
            if t > s + 1:
                j = np.arange(s + 1, t)
                sweep = max(sweep, int((wa[j - 1] + wa[j] + of[j - 1]).max()))
            m_null = wd[t] + sweep
            sp = np.arange(s + 1, t + 1)
            split = np.maximum(wa[sp - 1] + need[sp, t], need[s, sp - 1]).min()
            need[s, t] = min(max(m_all, wabar[s - 1] + need[s + 1, t]), max(m_null, split))
    return need[1:L + 1, 1:L + 1]


def infeasible_fraction(L, M, wa, wabar, wdelta=None, of=None, ob=None):
    """Fraction of the (s <= t, m in 0..M) cells of one chain that are infeasible."""
    need = min_feasible_memory(L, wa, wabar, wdelta, of, ob)
    iu = np.triu_indices(L)
    return float(np.minimum(need[iu], M + 1).sum()) / (len(iu[0]) * (M + 1))


def select_plan(costs, L, m_budget):
    """Final step of the planner's loop over candidate intra-op plans (Section "Integrate Two
    Solvers"): among the chains b, the one with the shortest total time C_BP(1, L, m_b) at its
    own budget m_b; the smallest b on ties; (-1, INF) if no chain is feasible.  A budget above
    the table's M reads column M; a negative budget is infeasible.

    costs: list of per-chain tables as returned by solve_chain; m_budget: list of ints.
    """
    best_b, best = -1, INF
    for b, (table, m) in enumerate(zip(costs, m_budget)):
        if m < 0:
            continue
        M = table.shape[2] - 1
        value = int(table[0, L - 1, min(int(m), M)])
        if value < best:
            best_b, best = b, value
    return best_b, best


SLOT_MAX = (1 << 31) - 1


def discretize(sizes_bytes, budget_bytes, M):
    """Memory discretisation the paper inherits from Rotor without describing it: the device
    budget is cut into M equal slots and every size is rounded UP to whole slots, so that a
    schedule that fits in slots fits in bytes:  slots = ceil(size * M / budget), computed in
    exact integer arithmetic and clamped to 2^31 - 1.  Python ints, no overflow."""
    budget = int(budget_bytes)
    if budget <= 0 or M < 0:
        raise ValueError("budget must be positive")
    out = []
    for v in sizes_bytes:
        v = int(v)
        if v < 0:
            raise ValueError("negative size")
        out.append(min(SLOT_MAX, -((-v * M) // budget)))
    return out


def budget_sweep(base_budget, alpha_num, alpha_den, count):
    """Memory budgets of the planner's loop (Section "Integrate Two Solvers"): the budgets
    (1 + alpha)^n, n = 0..count-1, scaled by a base budget, with alpha = alpha_num / alpha_den:
    budget_n = floor(base * (1 + alpha)^n), exact (Python integers)."""
    base, num, den = int(base_budget), int(alpha_num), int(alpha_den)
    if base <= 0 or num < 0 or den <= 0 or count < 1:
        raise ValueError("bad sweep")
    return [base * (den + num) ** n // den ** n for n in range(count)]


def discretize_sweep(sizes_bytes, base_budget, alpha_num, alpha_den, count, M):
    """One profile cut into slots under every budget of the sweep: row n is discretize() of the
    profile under budget_n."""
    return [discretize(sizes_bytes, b, M) for b in budget_sweep(base_budget, alpha_num, alpha_den, count)]


# Node flags of the linearisation input (one byte per node).
PLACEHOLDER, COMMON_SEED, NON_DIFF, IN_PLACE, COMM = 1, 2, 4, 8, 16


def linearize(children, flags):
    """Network linearisation: the node groups that become the stages of a chain, written from the
    definitions of Sections "Linearization", "Common Node" and "Full Set of Linearization Rules".

    Nodes 0..n-1 are in topological order; children[v] lists the children of v; flags[v] is a
    bit set of PLACEHOLDER (network input/output, never examined), COMMON_SEED (a
    non-differentiable input such as an attention mask), NON_DIFF (non-differentiable operation
    such as getattr/getitem), IN_PLACE, COMM (communication operation).

    Common nodes (definition and lemma of "Common Node"): a seeded node; an examined node whose
    operation is non-differentiable; an examined node all of whose parents are common (a node
    without parents counts as such).  Common nodes and placeholders hold no dependencies.

    End of a node group (basic rule of "Linearization" plus the two sticking rules): examined
    node v ends a group exactly when
      (a) no dependency is outstanding once v has been appended, i.e. no edge u -> c runs from
          an examined, non-common node u before v to an examined node c after v, and
      (b) no child of v is an in-place or a communication operation (such children stay in the
          group of their parent).
    Groups are the runs of examined nodes up to and including each end; nodes after the last end
    form a final group.

    Returns (group index per node, -1 for placeholders; common flag per node; number of groups).
    """
    n = len(children)
    examined = [not (flags[v] & PLACEHOLDER) for v in range(n)]
    parents = [[u for u in range(n) if v in children[u]] for v in range(n)]
    common = [False] * n
    for v in range(n):      # parents come first in a topological order
        common[v] = bool(flags[v] & COMMON_SEED) or (
            examined[v] and (bool(flags[v] & NON_DIFF) or all(common[p] for p in parents[v])))

    def outstanding(v):
        return any(examined[u] and not common[u] and examined[c] and c > v
                   for u in range(v) for c in children[u])

    def sticks(v):
        return any(flags[c] & (IN_PLACE | COMM) for c in children[v])

    group = [-1] * n
    ngroups, open_group = 0, False
    for v in range(n):
        if not examined[v]:
            continue
        group[v] = ngroups
        open_group = True
        if not outstanding(v) and not sticks(v):
            ngroups += 1
            open_group = False
    if open_group:
        ngroups += 1
    return group, common, ngroups
