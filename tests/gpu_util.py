"""Helpers shared by the GPU parity tests."""
import numpy as np


def oracle_tables(oracle_mod, batch, b, nthreads=1):
    """Oracle tables of chain b in the library's row order: (cost [rows, M+1], choice [rows, M+1])."""
    cost, choice = oracle_mod.solve_chain(batch.L, batch.M, *batch.chain(b), nthreads=nthreads)
    iu = np.triu_indices(batch.L)            # ordered by s, then t: the library's row order
    return cost[iu], choice[iu]


def assert_tables_equal(oracle_mod, batch, sol, nthreads=1, chains=None):
    """Bit-exact comparison of every cell (cost and recorded candidate) of the chosen chains."""
    M = batch.M
    for b in (range(batch.B) if chains is None else chains):
        want_cost, want_pick = oracle_tables(oracle_mod, batch, b, nthreads)
        got_cost = sol.cost[b, :, :M + 1].cpu().numpy()
        got_pick = sol.arg[b, :, :M + 1].cpu().numpy()
        bad = np.argwhere(got_cost != want_cost)
        assert bad.size == 0, f"{batch.name} chain {b}: {len(bad)} cost cells differ, first (row, m) = {bad[0]}, " \
                              f"got {got_cost[tuple(bad[0])]} want {want_cost[tuple(bad[0])]}"
        bad = np.argwhere(got_pick != want_pick)
        assert bad.size == 0, f"{batch.name} chain {b}: {len(bad)} arg cells differ, first (row, m) = {bad[0]}, " \
                              f"got {got_pick[tuple(bad[0])]} want {want_pick[tuple(bad[0])]}"
