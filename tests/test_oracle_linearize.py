"""Pins of the oracle's network linearisation (Sections "Linearization", "Common Node", "Full Set of
Linearization Rules"): three graphs cut by hand, and on random DAGs a last-use sweep and the
common-node lemma as a fixed point, both written differently from the oracle."""
import random

import pytest

P, SEED, NOND, INPL, COMM = 1, 2, 4, 8, 16


def _cuts_by_last_use(children, flags, common):
    """Where groups end, stated differently from the oracle (which scans edges per node): every
    examined, non-common node holds its dependencies until its LAST examined child has been
    appended, so the pool is empty after position v iff the running maximum of those last uses
    over the nodes before v does not pass v.  One forward sweep with a running maximum."""
    n = len(children)
    cuts, horizon = [], -1          # horizon: latest position at which a dependency of an earlier node ends
    for v in range(n):
        if flags[v] & P:
            continue
        sticky = any(flags[c] & (INPL | COMM) for c in children[v])
        if horizon <= v and not sticky:
            cuts.append(v)
        if not common[v]:
            horizon = max([horizon] + [c for c in children[v] if not flags[c] & P])
    return cuts


def _common_by_fixpoint(children, flags):
    """Lemma of Section "Common Node" as a fixed point over the whole graph."""
    n = len(children)
    parents = [[u for u in range(n) if v in children[u]] for v in range(n)]
    common = [bool(flags[v] & SEED) for v in range(n)]
    changed = True
    while changed:
        changed = False
        for v in range(n):
            if common[v] or flags[v] & P:
                continue
            if flags[v] & NOND or all(common[p] for p in parents[v]):
                common[v] = changed = True
    return common


def test_residual_blocks_by_hand(oracle_mod):
    """input -> stem -> [conv, conv, add(skip)] x 2 -> head -> output.  The skip edge keeps a block
    together; groups end at the stem, at each add, and at the head."""
    #            0:in 1:stem 2:conv 3:conv 4:add 5:conv 6:conv 7:add 8:head 9:out
    children = [[1], [2, 4], [3], [4], [5, 7], [6], [7], [8], [9], []]
    flags = [P, 0, 0, 0, 0, 0, 0, 0, 0, P]
    group, common, n = oracle_mod.linearize(children, flags)
    assert group == [-1, 0, 1, 1, 1, 2, 2, 2, 3, -1] and n == 4 and not any(common)


def test_attention_mask_is_a_common_node(oracle_mod):
    """A mask input used by every layer glues the layers into one group unless it is labelled
    common; getitem on the mask propagates the label (lemma), the layers then separate."""
    #            0:x 1:mask 2:getitem(mask) 3:layer1 4:layer2 5:layer3 6:out
    children = [[3], [2], [3, 4, 5], [4], [5], [6], []]
    plain = [P, P, 0, 0, 0, 0, P]
    group, common, n = oracle_mod.linearize(children, plain)
    assert n == 2 and group[2:6] == [0, 1, 1, 1]      # getitem alone (nothing pending yet), then all layers
    seeded = [P, P | SEED, 0, 0, 0, 0, P]
    group, common, n = oracle_mod.linearize(children, seeded)
    assert common[2] and not common[3] and group[3:6] == [group[3], group[3] + 1, group[3] + 2]
    nondiff = [P, P, NOND, 0, 0, 0, P]          # the operation itself is non-differentiable
    assert oracle_mod.linearize(children, nondiff)[0] == group


def test_in_place_and_communication_children_stick_to_their_parent(oracle_mod):
    #            0:in 1:bn 2:relu_(in-place) 3:linear 4:all_reduce(comm) 5:next 6:out
    children = [[1], [2], [3], [4], [5], [6], []]
    flags = [P, 0, INPL, 0, COMM, 0, P]
    group, _, n = oracle_mod.linearize(children, flags)
    assert group == [-1, 0, 0, 1, 1, 2, -1] and n == 3
    assert oracle_mod.linearize(children, [P, 0, 0, 0, 0, 0, P])[2] == 5


@pytest.mark.parametrize("seed", range(12))
def test_random_dags_against_the_definition(oracle_mod, seed):
    rng = random.Random(seed)
    n = rng.randrange(6, 40)
    children = [[] for _ in range(n)]
    for v in range(1, n):                                   # every node gets a parent: connected, topological
        for u in {rng.randrange(max(0, v - 5), v) for _ in range(rng.choice([1, 1, 2, 3]))}:
            children[u].append(v)
    flags = [0] * n
    for v in range(n):
        if not any(v in children[u] for u in range(n)):
            flags[v] = P | (SEED if rng.random() < 0.4 else 0)     # sources are inputs, some are masks
        elif not children[v]:
            flags[v] = P                                            # sinks are outputs
        else:
            r = rng.random()
            flags[v] = NOND if r < 0.1 else INPL if r < 0.2 else COMM if r < 0.27 else 0
    group, common, ngroups = oracle_mod.linearize(children, flags)
    assert common == [c and not (flags[v] & P and not flags[v] & SEED) for v, c in
                      enumerate(_common_by_fixpoint(children, flags))]
    cuts = _cuts_by_last_use(children, flags, common)
    examined = [v for v in range(n) if not flags[v] & P]
    want, g = {}, 0
    for v in examined:
        want[v] = g
        if v in cuts:
            g += 1
    assert [group[v] for v in examined] == [want[v] for v in examined]
    assert ngroups == (max(want.values()) + 1 if want else 0)
    assert all(group[v] == -1 for v in range(n) if flags[v] & P)
