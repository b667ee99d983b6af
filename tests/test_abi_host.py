"""Host-side checks of the C ABI: exported symbols, layout helpers, error codes and
ckpt_schedule (which runs on the host).  No GPU compute is called here."""
import ctypes
import os
import re

import numpy as np
import pytest

from persistent_bruteforce import simulate
from workloads import make_config, random_chain_batch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def amd():
    import paper_2302_02599_amd as amd
    if not os.path.exists(amd.lib_path()):
        from paper_2302_02599_amd.build import build_library
        build_library()
    amd.load_library()
    return amd


def test_library_exports_every_declared_symbol(amd):
    header = open(os.path.join(ROOT, "include", "ckpt_dp.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(ckpt_[a-z_]+)\s*\(", header))
    assert {"ckpt_solve_batched", "ckpt_schedule", "ckpt_workspace_bytes", "ckpt_row_index"} <= names
    lib = ctypes.CDLL(amd.lib_path())
    for n in sorted(names):
        assert hasattr(lib, n), n


def test_layout_helpers(amd):
    assert amd.ckpt_row_pitch(0) == 64 and amd.ckpt_row_pitch(63) == 64 and amd.ckpt_row_pitch(64) == 128
    assert amd.ckpt_row_pitch(4096) == 4160 and amd.ckpt_row_pitch(-1) == 0
    for L in (1, 2, 7, 24):
        seen = []
        for s in range(1, L + 1):
            for t in range(s, L + 1):
                seen.append(amd.ckpt_row_index(L, s, t))
        assert seen == list(range(L * (L + 1) // 2))      # ordered by s then t, no gaps
        assert amd.ckpt_table_rows(L) == len(seen)
    assert amd.ckpt_row_index(5, 3, 2) == -1 and amd.ckpt_row_index(5, 0, 2) == -1 and amd.ckpt_row_index(5, 1, 6) == -1
    assert amd.ckpt_table_elems(8, 64, 2) == 2 * 36 * 128
    assert amd.ckpt_workspace_bytes(0, 4, 1) == 0 and amd.ckpt_workspace_bytes(8, 64, 1) > 0


def test_solve_rejects_bad_arguments_before_touching_the_gpu(amd):
    lib = amd.load_library()
    from paper_2302_02599_amd.binding import _Chains
    ch = _Chains(256, 256, 256, 256, None, None, None)
    f = lib.ckpt_solve_batched
    assert f(None, 4, 8, 1, None, 256, 256, 256) == -1
    assert f(ctypes.byref(ch), 0, 8, 1, None, 256, 256, 256) == -1
    assert f(ctypes.byref(ch), 4, -1, 1, None, 256, 256, 256) == -1
    assert f(ctypes.byref(ch), 4, 8, 0, None, 256, 256, 256) == -1
    assert f(ctypes.byref(ch), 255, 8, 1, None, 256, 256, 256) == -2          # arg is one byte
    assert f(ctypes.byref(ch), 254, 2 ** 16, 1, None, 256, 256, 256) == -2    # chain table of 4 GiB or more
    assert f(ctypes.byref(ch), 4, 8, 65536, None, 256, 256, 256) == -2         # more chains than a grid dimension
    assert f(ctypes.byref(ch), 4, 8, 1, None, 260, 256, 256) == -1            # misaligned table
    assert f(ctypes.byref(ch), 4, 8, 1, None, None, 256, 256) == -1
    ch2 = _Chains(256, None, 256, 256, None, None, None)
    assert f(ctypes.byref(ch2), 4, 8, 1, None, 256, 256, 256) == -1
    assert lib.ckpt_strerror(-2) == b"size limit exceeded"


def _arg_table_from_oracle(amd, choice, L, M):
    pitch = amd.ckpt_row_pitch(M)
    tab = np.full((amd.ckpt_table_rows(L), pitch), 0xEE, np.uint8)   # padding holds junk
    for s in range(1, L + 1):
        for t in range(s, L + 1):
            tab[amd.ckpt_row_index(L, s, t), :M + 1] = choice[s - 1, t - 1]
    return tab


@pytest.mark.parametrize("which", ["cfg0", "cfg1", "rand"])
def test_schedule_matches_oracle_and_simulator(amd, oracle_mod, which):
    batch = {"cfg0": lambda: make_config(0), "cfg1": lambda: make_config(1),
             "rand": lambda: random_chain_batch(11, 70, 1, 31, overheads=True, own_wdelta=True)}[which]()
    L, M = batch.L, batch.M
    ch = batch.chain(0)
    cost, choice = oracle_mod.solve_chain(L, M, *ch)
    tab = _arg_table_from_oracle(amd, choice, L, M)
    n_checked = 0
    for (s, t) in [(1, L), (2, L), (1, L - 1), (L // 2, L // 2)]:
        for m in range(0, M + 1, max(1, M // 25)):
            if cost[s - 1, t - 1, m] >= oracle_mod.INF:
                with pytest.raises(amd.CkptError) as e:
                    amd.ckpt_schedule(tab, ch[2], ch[3], L, M, s, t, m)
                assert e.value.code == -3
                continue
            ops = amd.ckpt_schedule(tab, ch[2], ch[3], L, M, s, t, m)
            assert ops == oracle_mod.reconstruct(choice, ch[2], ch[3], s, t, m)
            time, peak = simulate(ops, s, t, *ch)
            assert time == cost[s - 1, t - 1, m] and peak <= m
            n_checked += 1
    assert n_checked > 10


def test_schedule_error_codes(amd, oracle_mod):
    batch = make_config(0)
    L, M = batch.L, batch.M
    ch = batch.chain(0)
    _, choice = oracle_mod.solve_chain(L, M, *ch)
    tab = _arg_table_from_oracle(amd, choice, L, M)
    full = amd.ckpt_schedule(tab, ch[2], ch[3], L, M, 1, L, M)
    # a budget above the table's M reads column M, as in the batched walk and the plan selection
    assert amd.ckpt_schedule(tab, ch[2], ch[3], L, M, 1, L, M + 1) == full
    assert amd.ckpt_schedule(tab, ch[2], ch[3], L, M, 1, L, 2 ** 31 - 1) == full
    for bad in [dict(s=0), dict(t=L + 1), dict(s=3, t=2), dict(m_budget=-1)]:
        kw = dict(s=1, t=L, m_budget=M); kw.update(bad)
        with pytest.raises(amd.CkptError) as e:
            amd.ckpt_schedule(tab, ch[2], ch[3], L, M, kw["s"], kw["t"], kw["m_budget"])
        assert e.value.code == -1
    with pytest.raises(amd.CkptError) as e:
        amd.ckpt_schedule(tab, ch[2], ch[3], L, M, 1, L, M, ops_cap=len(full) - 1)
    assert e.value.code == -4
    assert amd.ckpt_schedule(tab, ch[2], ch[3], L, M, 1, L, M, ops_cap=len(full)) == full
    broken = tab.copy()
    broken[amd.ckpt_row_index(L, 1, L), M] = L + 3          # candidate outside [s, t]
    with pytest.raises(amd.CkptError) as e:
        amd.ckpt_schedule(broken, ch[2], ch[3], L, M, 1, L, M)
    assert e.value.code == -7


def test_block_indices_host_matches_oracle(amd, oracle_mod):
    """Section "Code generation": block index per stage from the whole-chain operation list; every
    budget of cfg 0 and cfg 1, and every persistent schedule of short chains."""
    from persistent_bruteforce import flatten, trees
    for cfg in (0, 1):
        batch = make_config(cfg)
        L, M = batch.L, batch.M
        ch = batch.chain(0)
        cost, choice = oracle_mod.solve_chain(L, M, *ch)
        tab = _arg_table_from_oracle(amd, choice, L, M)
        kinds = set()
        for m in range(M + 1):
            if cost[0, L - 1, m] >= oracle_mod.INF:
                continue
            ops = amd.ckpt_schedule(tab, ch[2], ch[3], L, M, 1, L, m)
            got = amd.ckpt_block_indices(ops, L)
            assert got == oracle_mod.block_indices(ops, L), m
            kinds.add(tuple(got[0]))
        assert len(kinds) > 3
    for L in (1, 2, 3, 4, 5):
        for tree in trees(1, L):
            ops = flatten(tree)
            assert amd.ckpt_block_indices(ops, L) == oracle_mod.block_indices(ops, L)


def test_block_indices_error_codes(amd):
    A, C, N, B = 0, 1, 2, 3
    ok = [(C, 1), (N, 2), (A, 3), (B, 3), (A, 1), (A, 2), (B, 2), (B, 1)]
    assert amd.ckpt_block_indices(ok, 3) == ([0, 0, -1], 1)
    for bad in ([(A, 1), (B, 1)],                            # shorter than the chain
                [(A, 1), (N, 2), (A, 3), (B, 3)],            # F_null after a kept stage
                [(N, 1), (A, 2), (B, 2)],                    # F_null^1 has nothing to continue
                [(A, 2), (A, 1), (B, 2)],                    # stages out of order
                [(A, 1), (A, 2), (A, 2)],                    # no B^L after the forward sweep
                [(A, 1), (B, 2), (B, 2)]):
        with pytest.raises(amd.CkptError) as e:
            amd.ckpt_block_indices(bad, 2 if len(bad) == 3 else 3 if len(bad) > 3 else 2)
        assert e.value.code == -7, bad
    lib = amd.load_library()
    assert lib.ckpt_block_indices(None, 3, 3, None) == -1
    assert lib.ckpt_block_indices_batched(None, 4, 256, 3, 1, None, 256, 256) == -1
    assert lib.ckpt_block_indices_batched(256, 4, 256, 255, 1, None, 256, 256) == -2


def test_options_are_validated_on_the_host(amd):
    lib = amd.load_library()
    from paper_2302_02599_amd.binding import _Chains, _SolveOpts
    ch = _Chains(256, 256, 256, 256, None, None, None)
    f = lib.ckpt_solve_batched_opts
    for groups, split in ((-1, 0), (5, 0), (0, 3), (0, 8), (0, -1)):
        o = _SolveOpts()
        o.groups, o.list_split = groups, split
        assert f(ctypes.byref(ch), 4, 8, 1, None, 256, 256, 256, ctypes.byref(o)) == -1, (groups, split)
    for field, bad in (("row_launches", 2), ("row_launches", -1), ("frontier", 3), ("frontier", -1)):
        o = _SolveOpts()
        setattr(o, field, bad)
        assert f(ctypes.byref(ch), 4, 8, 1, None, 256, 256, 256, ctypes.byref(o)) == -1, (field, bad)
    o = _SolveOpts()
    o.groups = 3
    o.side_streams[1] = 4096                                  # second side stream given, first missing
    assert f(ctypes.byref(ch), 4, 8, 1, None, 256, 256, 256, ctypes.byref(o)) == -1
    assert lib.ckpt_init(64) == -2
    assert lib.ckpt_strerror(-8).startswith(b"helper streams")


def test_schedule_worst_case_length_fits_default_capacity(amd):
    # a table that always splits at s' = t gives the longest sequence: L(L+1)/2 + L operations
    L, M = 9, 3
    pitch = amd.ckpt_row_pitch(M)
    tab = np.zeros((amd.ckpt_table_rows(L), pitch), np.uint8)
    for s in range(1, L + 1):
        for t in range(s, L + 1):
            tab[amd.ckpt_row_index(L, s, t), :] = t
    ops = amd.ckpt_schedule(tab, np.zeros(L + 1, np.int32), np.zeros(L, np.int32), L, M, 1, L, M)
    assert len(ops) == L * (L + 1) // 2 + L


def test_planner_steps_reject_bad_arguments_before_touching_the_gpu(amd):
    lib = amd.load_library()
    from paper_2302_02599_amd.binding import _Chains
    assert lib.ckpt_select_plan(None, 4, 8, 1, 256, None, 256) == -1
    assert lib.ckpt_select_plan(256, 4, 8, 1, 256, None, None) == -1
    assert lib.ckpt_select_plan(256, 0, 8, 1, 256, None, 256) == -1
    assert lib.ckpt_select_plan(256, 255, 8, 1, 256, None, 256) == -2
    outs = _Chains(None, None, 256, 256, None, None, None)
    f = lib.ckpt_discretize
    assert f(256, 256, None, None, None, 256, 4, 8, 1, None, None) == -1
    assert f(None, 256, None, None, None, 256, 4, 8, 1, None, ctypes.byref(outs)) == -1
    assert f(256, 256, 256, None, None, 256, 4, 8, 1, None, ctypes.byref(outs)) == -1   # input without its output
    assert f(256, 256, None, None, None, 256, 4, (1 << 20) + 1, 1, None, ctypes.byref(outs)) == -2
    g = lib.ckpt_schedule_batched
    assert g(256, 256, 256, 4, 8, 1, 256, None, 256, 10, 256, None) == -1               # no workspace
    assert g(256, 256, 256, 4, 8, 1, 256, None, 256, 10, 256, 264) == -1                # misaligned workspace
    assert g(256, 256, 256, 4, 8, 1, 256, None, 256, -1, 256, 256) == -1
    assert amd.ckpt_schedule_workspace_bytes(8, 3) == 3 * 18 * 16 and amd.ckpt_schedule_workspace_bytes(0, 3) == 0
    h = lib.ckpt_simulate_batched
    chains = _Chains(256, 256, 256, 256, None, None, None)
    assert h(ctypes.byref(chains), 4, 1, None, 10, 256, None, 256, 256, 256) == -1              # no list
    assert h(ctypes.byref(chains), 0, 1, 256, 10, 256, None, 256, 256, 256) == -1
    assert h(ctypes.byref(chains), 255, 1, 256, 10, 256, None, 256, 256, 256) == -2
    w = lib.ckpt_discretize_sweep
    assert w(256, 256, None, None, None, 1000, 1, 10, 4, 4, 8, None, None, None) == -1           # no outputs
    assert w(256, 256, None, None, None, 0, 1, 10, 4, 4, 8, None, None, ctypes.byref(outs)) == -1
    assert w(256, 256, None, None, None, 1000, 1, 10, 17, 4, 8, None, None, ctypes.byref(outs)) == -2


def test_budget_sweep_on_the_host(amd, oracle_mod):
    """Host arithmetic of the sweep against the oracle's exact integers."""
    rng = np.random.default_rng(12)
    cases = [(1000, 1, 10, 10), (80 << 30, 1, 10, 10), (1, 0, 1, 16), (3, 1, 1, 16), (7, 1, 2, 4),
             ((1 << 62) - 5, 0, 7, 3), (12345678901, 3, 20, 10)]
    for _ in range(200):
        cases.append((int(rng.integers(1, 1 << 45)), int(rng.integers(0, 60)), int(rng.integers(1, 101)),
                      int(rng.integers(1, 11))))
    lib = amd.load_library()
    out = np.zeros(32, np.int64)
    fits = 0
    for base, num, den, count in cases:
        want = oracle_mod.budget_sweep(base, num, den, count)
        if want[-1] < 1 << 63:
            assert amd.ckpt_budget_sweep(base, num, den, count) == want, (base, num, den, count)
            fits += 1
        else:   # a budget that does not fit 64 bits is refused, not wrapped
            assert lib.ckpt_budget_sweep(base, num, den, count, out.ctypes.data) == -2, (base, num, den, count)
    assert fits > 100
    for args, want in (((0, 1, 10, 3), -1), ((5, -1, 10, 3), -1), ((5, 1, 0, 3), -1), ((5, 1, 10, 0), -1),
                       ((5, 1, 10, 17), -2), ((1 << 62, 1, 1, 3), -2), ((1 << 40, 1 << 30, 1, 16), -2),
                       ((1 << 40, 0, 1 << 30, 16), -2)):
        assert lib.ckpt_budget_sweep(*args, out.ctypes.data) == want, args
    assert lib.ckpt_budget_sweep(5, 1, 10, 3, None) == -1
