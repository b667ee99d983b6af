"""Pins of the oracle's checkpoint block indices (oracle.block_indices, Section "Code generation").

Hand-derived indices for the worked example; on every persistent schedule of short chains the
indices read off the DECOMPOSITION TREE (no operation list involved: the root of a segment
either keeps stage s and goes on with s+1..t, or checkpoints s..s'-1 as one block and goes on
with s'..t); on the recurrence's own schedules, the same walk over the table of recorded choices.
"""
import os

import numpy as np
import pytest

import persistent_bruteforce as bf
from workloads import make_config, random_chain_batch

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
KIND = {"A": 0, "C": 1, "N": 2, "B": 3}


def blocks_of_tree(tree, L):
    """Block index per stage from the tree's spine: ("all", s, rest) keeps stage s, ("ck", s, s',
    right, left) makes s..s'-1 one block and continues in `right`; a leaf keeps its stage."""
    block, n = [None] * L, 0
    while True:
        if tree[0] == "leaf":
            block[tree[1] - 1] = -1
            break
        if tree[0] == "all":
            block[tree[1] - 1] = -1
            tree = tree[2]
        else:
            _, s, sp, right, _left = tree
            for j in range(s, sp):
                block[j - 1] = n
            n += 1
            tree = right
    return block, n


def test_hand_derived_blocks(oracle_mod):
    rows = []
    with open(os.path.join(GOLDEN, "worked_example_L3_blocks.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            m, ops, blocks, n = [p.strip() for p in line.split("|")]
            rows.append(([(KIND[o[0]], int(o[1:])) for o in ops.split()], [int(v) for v in blocks.split()], int(n)))
    assert len(rows) == 5
    for ops, blocks, n in rows:
        assert oracle_mod.block_indices(ops, 3) == (blocks, n)


@pytest.mark.parametrize("L", [1, 2, 3, 4, 5, 6])
def test_every_persistent_schedule_against_its_tree(oracle_mod, L):
    count = 0
    for tree in bf.trees(1, L):
        assert oracle_mod.block_indices(bf.flatten(tree), L) == blocks_of_tree(tree, L)
        count += 1
    assert count == [1, 2, 6, 22, 90, 394][L - 1]


@pytest.mark.parametrize("cfg", [0, 1])
def test_blocks_of_the_recurrence_schedules(oracle_mod, cfg):
    """Walk of the recorded choices along the spine (no operation list) against block_indices of
    the reconstructed list; and the invariants: blocks are runs of consecutive stages numbered in
    chain order, the last stage is never inside a block (its leaf runs F_all)."""
    batch = make_config(cfg)
    L, M = batch.L, batch.M
    ch = batch.chain(0)
    wa, wabar = ch[2], ch[3]
    cost, choice = oracle_mod.solve_chain(L, M, *ch)
    seen = set()
    for m in range(M + 1):
        if cost[0, L - 1, m] >= oracle_mod.INF:
            continue
        want, n, s, mm = [None] * L, 0, 1, m
        while s <= L:
            k = int(choice[s - 1, L - 1, mm])
            if k == s:
                want[s - 1] = -1
                mm -= int(wabar[s - 1])
                s += 1
            else:
                for j in range(s, k):
                    want[j - 1] = n
                n += 1
                mm -= int(wa[k - 1])
                s = k
        got, ngot = oracle_mod.block_indices(oracle_mod.reconstruct(choice, wa, wabar, 1, L, m), L)
        assert (got, ngot) == (want, n), m
        assert got[-1] == -1
        inside = [b for b in got if b >= 0]
        assert inside == sorted(inside) and set(inside) == set(range(n))
        seen.add(tuple(got))
    assert len(seen) > 3


def test_lists_that_cannot_be_annotated(oracle_mod):
    with pytest.raises(ValueError):
        oracle_mod.block_indices([(0, 1), (3, 1)], 2)                    # stage 2 never runs
    with pytest.raises(ValueError):
        oracle_mod.block_indices([(0, 1), (2, 2), (0, 3)], 3)            # F_null^2 after a kept stage
    with pytest.raises(ValueError):
        oracle_mod.block_indices([(2, 1)], 1)                            # F_null^1 has no block to continue
