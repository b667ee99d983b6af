"""The library's host linearisation equals the oracle's on hand-made and random DAGs."""
import os
import random

import numpy as np
import pytest

P, SEED, NOND, INPL, COMM = 1, 2, 4, 8, 16


@pytest.fixture(scope="module")
def amd():
    import paper_2302_02599_amd as amd
    if not os.path.exists(amd.lib_path()):
        from paper_2302_02599_amd.build import build_library
        build_library()
    amd.load_library()
    return amd


def _random_dag(rng, n):
    children = [[] for _ in range(n)]
    for v in range(1, n):
        for u in {rng.randrange(max(0, v - 6), v) for _ in range(rng.choice([1, 1, 2, 3]))}:
            children[u].append(v)
    flags = [0] * n
    has_parent = [False] * n
    for u in range(n):
        for c in children[u]:
            has_parent[c] = True
    for v in range(n):
        if not has_parent[v]:
            flags[v] = P | (SEED if rng.random() < 0.4 else 0)
        elif not children[v]:
            flags[v] = P
        else:
            r = rng.random()
            flags[v] = NOND if r < 0.1 else INPL if r < 0.2 else COMM if r < 0.27 else 0
    return children, flags


def test_hand_made_graphs(amd, oracle_mod):
    cases = [
        ([[1], [2, 4], [3], [4], [5, 7], [6], [7], [8], [9], []], [P, 0, 0, 0, 0, 0, 0, 0, 0, P]),
        ([[3], [2], [3, 4, 5], [4], [5], [6], []], [P, P | SEED, 0, 0, 0, 0, P]),
        ([[1], [2], [3], [4], [5], [6], []], [P, 0, INPL, 0, COMM, 0, P]),
        ([], []),
        ([[]], [0]),
    ]
    for children, flags in cases:
        assert amd.ckpt_linearize(children, flags) == oracle_mod.linearize(children, flags)
    assert amd.ckpt_linearize(cases[0][0], cases[0][1])[0] == [-1, 0, 1, 1, 1, 2, 2, 2, 3, -1]


@pytest.mark.parametrize("seed", range(25))
def test_random_dags(amd, oracle_mod, seed):
    rng = random.Random(1000 + seed)
    children, flags = _random_dag(rng, rng.randrange(2, 400))
    assert amd.ckpt_linearize(children, flags) == oracle_mod.linearize(children, flags)


def test_rejects_edges_that_are_not_forward(amd):
    with pytest.raises(amd.CkptError) as e:
        amd.ckpt_linearize([[1], [0]], [0, 0])
    assert e.value.code == -1
    with pytest.raises(amd.CkptError):
        amd.ckpt_linearize([[5]], [0])
    lib = amd.load_library()
    assert lib.ckpt_linearize(3, None, None, None, None, None) == -1


def test_groups_become_a_chain_the_solver_accepts(amd, oracle_mod):
    """End to end on the host side: a residual network's groups give per-stage times and sizes;
    the oracle solves the resulting chain (one stage per group)."""
    blocks = 6
    children, flags = [[1]], [P]                       # input
    children.append([2, 4]); flags.append(0)           # stem feeds block 1 and its skip
    v = 2
    for k in range(blocks):
        children += [[v + 1], [v + 2], [v + 3, v + 5] if k < blocks - 1 else [v + 3]]
        flags += [0, 0, 0]
        v += 3
    children.append([]); flags.append(P)
    group, _, n = amd.ckpt_linearize(children, flags)
    assert n == blocks + 1
    rng = np.random.default_rng(0)
    node_time = rng.integers(5, 50, len(children))
    uf = np.array([sum(node_time[u] for u in range(len(children)) if group[u] == g) for g in range(n)], np.int32)
    wa = np.ones(n + 1, np.int32) * 2
    wabar = np.array([2 * sum(1 for u in range(len(children)) if group[u] == g) for g in range(n)], np.int32)
    cost, _ = oracle_mod.solve_chain(n, 40, uf, 2 * uf, wa, wabar)
    assert cost[0, n - 1, 40] == 3 * uf.sum()
