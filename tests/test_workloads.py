"""The synthetic workloads have the stated shapes, ranges and structure."""
import numpy as np
import pytest

from workloads import CONFIGS, make_config


@pytest.mark.parametrize("idx", range(5))
def test_shapes_and_basic_structure(idx):
    b = make_config(idx)
    c = CONFIGS[idx]
    assert (b.L, b.M, b.B) == (c["L"], c["M"], c["B"])
    assert b.uf.shape == (b.B, b.L) and b.wa.shape == (b.B, b.L + 1) and b.wabar.shape == (b.B, b.L)
    assert all(a.dtype == np.int32 for a in (b.uf, b.ub, b.wa, b.wabar))
    assert (b.uf >= 1).all() and (b.wa >= 1).all()
    if idx != 2:                                   # cfg2 adds independent noise after the shard division
        assert (b.ub >= 2 * b.uf).all()
    assert (b.wabar >= b.wa[:, 1:]).all()          # abar^i contains a^i
    # costs stay far below the 2^30 sentinel even if every forward were rerun per stage
    assert int(b.L * b.uf.astype(np.int64).sum(axis=1).max() + b.ub.astype(np.int64).sum(axis=1).max()) < 2 ** 30
    again = make_config(idx)
    assert all((x == y).all() for x, y in zip(b.dense(), again.dense()))


def test_cfg1_mlp_twice_attention():
    b = make_config(1)
    assert (b.uf[0, 1::2] == 2 * b.uf[0, 0::2]).all()
    assert b.uf.min() >= 200 and b.uf.max() <= 2000


def test_cfg2_shard_factors():
    b = make_config(2)
    # chains with the same shard factor share sizes; higher factor -> smaller sizes
    assert (b.wa[0] == b.wa[4]).all() and (b.wa[1] == b.wa[5]).all()
    assert (b.wa[3] <= b.wa[2]).all() and (b.wa[2] <= b.wa[1]).all() and (b.wa[1] <= b.wa[0]).all()
    assert not (b.uf[0] == b.uf[4]).all()          # fresh communication noise per chain


def test_cfg4_infeasible_fraction(oracle_mod):
    b = make_config(4)
    for i in range(b.B):
        frac = oracle_mod.infeasible_fraction(b.L, b.M, b.wa[i], b.wabar[i])
        assert abs(frac - 0.30) <= 0.01, (i, frac)


def test_min_feasible_memory_matches_table(oracle_mod):
    b = make_config(1)
    cost, _ = oracle_mod.solve_chain(b.L, b.M, *b.chain(0))
    need = oracle_mod.min_feasible_memory(b.L, b.wa[0], b.wabar[0])
    for s in range(1, b.L + 1):
        for t in range(s, b.L + 1):
            row = cost[s - 1, t - 1]
            first = int(np.argmax(row < oracle_mod.INF)) if (row < oracle_mod.INF).any() else b.M + 1
            assert first == min(int(need[s - 1, t - 1]), b.M + 1)
