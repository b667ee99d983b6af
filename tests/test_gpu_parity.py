"""GPU parity: the HIP tables equal the CPU oracle's bit for bit (cost and recorded candidate).

All calls go through the C ABI (paper_2302_02599_amd.binding).  Integer work: the bar is
exact equality of every cell."""
import numpy as np
import pytest

from gpu_util import assert_tables_equal
from persistent_bruteforce import simulate
from workloads import ChainBatch, make_config, random_chain_batch

pytestmark = pytest.mark.gpu
_full = {}


@pytest.fixture(scope="module")
def amd():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2302_02599_amd as amd
    amd.load_library()          # raises if the HIP library is not built: there is no fallback
    return amd


@pytest.mark.parametrize("cfg", [0, 1, 2])
def test_configs_small(amd, oracle_mod, cfg):
    batch = make_config(cfg)
    print(f"case {batch.name}", flush=True)
    assert_tables_equal(oracle_mod, batch, amd.solve(batch), nthreads=8)


@pytest.mark.parametrize("L,M,B,seed,ovh,wd,zero", [
    (1, 0, 1, 1, False, False, False), (1, 40, 3, 2, True, True, False),
    (2, 63, 2, 3, True, False, False), (3, 64, 2, 4, False, True, False),
    (7, 65, 3, 5, True, True, False), (8, 127, 2, 6, False, False, True),
    (9, 200, 2, 7, True, True, False), (13, 129, 2, 8, True, False, False),
    (16, 255, 2, 9, False, False, False), (17, 256, 3, 10, True, True, True),
    (23, 300, 2, 11, True, True, False), (31, 513, 2, 12, False, True, False),
    (33, 97, 5, 13, True, False, False), (40, 1, 2, 14, False, False, False),
    (50, 130, 2, 15, True, True, False), (57, 66, 3, 16, False, False, False), (71, 190, 1, 17, True, True, False),
    (64, 64, 2, 18, False, True, False), (100, 70, 1, 19, True, False, False),
    (254, 130, 1, 20, True, True, False), (192, 300, 2, 21, False, False, False),
])
def test_ragged_shapes(amd, oracle_mod, L, M, B, seed, ovh, wd, zero):
    """Chain lengths and budgets that are not multiples of any tile, incl. M = 0 and L = 1."""
    batch = random_chain_batch(L, M, B, seed, size_hi=max(2, min(9, (M + 8) // 8)), overheads=ovh,
                               own_wdelta=wd, zero_sizes=zero)
    print(f"case {batch.name}", flush=True)
    assert_tables_equal(oracle_mod, batch, amd.solve(batch), nthreads=4)


@pytest.mark.parametrize("seed", range(16))
def test_random_shapes(amd, oracle_mod, seed):
    """Seeded sweep over chain lengths, budgets, batch sizes and optional arrays."""
    rng = np.random.default_rng(9000 + seed)
    L = int(rng.integers(1, 90))
    M = int(rng.integers(0, 700))
    B = int(rng.integers(1, 6))
    batch = random_chain_batch(L, M, B, 500 + seed, size_hi=int(rng.integers(1, 12)),
                               time_hi=int(rng.integers(2, 3000)), overheads=bool(rng.integers(2)),
                               own_wdelta=bool(rng.integers(2)), zero_sizes=bool(rng.integers(2)))
    print(f"case {batch.name} size_hi etc. seed {seed}", flush=True)
    assert_tables_equal(oracle_mod, batch, amd.solve(batch), nthreads=4)


@pytest.mark.parametrize("L,M,B,seed,size_hi", [
    (6, 70000, 2, 31, 9000),      # rows much wider than any tile of m
    (20, 20000, 1, 32, 1500),
    (40, 36000, 3, 33, 1200),     # large enough for the multi-stream schedule: three groups of one chain
    (32, 30000, 5, 35, 1000),     # four groups of 1, 1, 1 and 2 chains
    (10, 100, 700, 34, 9),        # more chains than threads of any block
    (254, 4096, 2, 36, 120),      # the longest chain the library takes, at the width of the benchmark
])
def test_wide_rows_and_many_chains(amd, oracle_mod, L, M, B, seed, size_hi):
    batch = random_chain_batch(L, M, B, seed, size_hi=size_hi, time_hi=5000, overheads=True, own_wdelta=True)
    print(f"case {batch.name}", flush=True)
    assert_tables_equal(oracle_mod, batch, amd.solve(batch), nthreads=8)


def test_everything_infeasible(amd, oracle_mod):
    batch = random_chain_batch(12, 3, 2, 21, size_hi=9)
    batch.wa += 5
    batch.wabar += 5
    sol = amd.solve(batch)
    assert_tables_equal(oracle_mod, batch, sol)
    assert (sol.cost[:, :, :batch.M + 1] == amd.CKPT_INF).all() and (sol.arg[:, :, :batch.M + 1] == 0).all()


def test_costs_saturate_at_the_sentinel(amd, oracle_mod):
    """Times large enough that long segments pass 2^30: those cells hold exactly the sentinel."""
    batch = random_chain_batch(6, 80, 2, 22, size_hi=5)
    batch.uf[:] = 150_000_000 + np.arange(6, dtype=np.int32)
    batch.ub[:] = 300_000_000 - np.arange(6, dtype=np.int32)
    sol = amd.solve(batch)
    assert_tables_equal(oracle_mod, batch, sol)
    root = sol.cost[0, amd.ckpt_row_index(6, 1, 6), batch.M].item()
    one = sol.cost[0, amd.ckpt_row_index(6, 2, 2), batch.M].item()
    assert root == amd.CKPT_INF and one == 450_000_000


def test_abar_smaller_than_a_is_flagged_and_follows_the_printed_formulas(amd, oracle_mod):
    """Outside the Theorem's model (abar contains a): the chains are flagged (bit 8); their tables
    are still what the printed formulas give -- formula conformance, not parity with an optimum."""
    rng = np.random.default_rng(23)
    L, M, B = 14, 90, 2
    batch = ChainBatch("abar_lt_a", L, M, B,
                       uf=rng.integers(1, 50, (B, L)).astype(np.int32), ub=rng.integers(1, 90, (B, L)).astype(np.int32),
                       wa=rng.integers(1, 9, (B, L + 1)).astype(np.int32), wabar=rng.integers(0, 6, (B, L)).astype(np.int32),
                       wdelta=rng.integers(0, 7, (B, L + 1)).astype(np.int32),
                       of=rng.integers(0, 4, (B, L)).astype(np.int32), ob=rng.integers(0, 4, (B, L)).astype(np.int32))
    batch.wabar[1] = np.maximum(batch.wabar[1], batch.wa[1, 1:])     # chain 1 is inside the model
    sol = amd.solve(batch, check=False)
    assert amd.ckpt_check_inputs(sol.workspace, L, M, B).tolist() == [8, 0]
    assert_tables_equal(oracle_mod, batch, sol)


def test_sizes_larger_than_the_budget(amd, oracle_mod):
    """A stage whose activation exceeds M + 1: shifts beyond the row stay in bounds and read as infeasible."""
    batch = random_chain_batch(10, 50, 2, 24, size_hi=6)
    batch.wa[:, 4] = 5000
    batch.wabar[:, 3] = 5003
    batch.wabar[:, 6] = 70
    assert_tables_equal(oracle_mod, batch, amd.solve(batch))


def test_bad_inputs_are_flagged_not_faulted(amd):
    import torch
    batch = random_chain_batch(9, 60, 3, 25)
    batch.uf[1, 3] = -7
    batch.wa[2, 2] = -3
    batch.wabar[2, 5] = (1 << 28) + 1
    sol = amd.solve(batch, check=False)
    flags = amd.ckpt_check_inputs(sol.workspace, batch.L, batch.M, batch.B)
    torch.cuda.synchronize()
    assert flags[0] == 0 and flags[1] & 1 and flags[2] & 1 and flags[2] & 4
    with pytest.raises(amd.CkptError):
        amd.solve(batch)


def test_two_solves_are_bit_identical(amd):
    batch = make_config(2)
    a, b = amd.solve(batch), amd.solve(batch)
    M = batch.M
    assert (a.cost[:, :, :M + 1] == b.cost[:, :, :M + 1]).all() and (a.arg[:, :, :M + 1] == b.arg[:, :, :M + 1]).all()


def _same_tables(a, b, M):
    return bool((a.cost[:, :, :M + 1] == b.cost[:, :, :M + 1]).all() and (a.arg[:, :, :M + 1] == b.arg[:, :, :M + 1]).all())


@pytest.mark.parametrize("which", ["cfg2", "wide"])
def test_tables_do_not_depend_on_the_schedule(amd, oracle_mod, which):
    """The same input under every work order the library can take: one stream or 2, 3, 4 groups of
    chains (the library's helper streams or the caller's), 1, 2 or 4 waves per list of splits
    in the block-product kernel, and the rows of a block diagonal in one launch or in seven.  Every variant must give the tables of the plain call, bit for bit
    (and those equal the oracle's, checked on one chain)."""
    import torch
    batch = make_config(2) if which == "cfg2" else \
        random_chain_batch(32, 30000, 5, 35, size_hi=1000, time_hi=5000, overheads=True)
    M = batch.M
    amd.ckpt_init()
    base = amd.solve(batch)
    assert_tables_equal(oracle_mod, batch, base, nthreads=8, chains=[batch.B - 1])
    own = [torch.cuda.Stream() for _ in range(3)]
    variants = [dict(groups=1), dict(groups=2), dict(groups=3), dict(groups=4),
                dict(groups=1, list_split=1), dict(groups=1, list_split=2), dict(groups=1, list_split=4),
                dict(groups=4, list_split=2), dict(groups=2, list_split=4),
                dict(groups=4, side_streams=[s.cuda_stream for s in own]),
                dict(groups=3, list_split=1, side_streams=[s.cuda_stream for s in own[:2]]),
                dict(row_launches=1), dict(groups=1, row_launches=1), dict(groups=4, row_launches=1, list_split=2),
                dict(frontier=1), dict(frontier=2), dict(groups=1, frontier=1), dict(groups=4, frontier=2, stagger=1),
                dict(groups=3, stagger=1, row_launches=1), dict(spin_limit=5000000)]
    for opts in variants:
        print(f"case {batch.name} {opts}", flush=True)
        other = amd.solve(batch, **opts)
        torch.cuda.synchronize()
        assert _same_tables(base, other, M), opts


def test_a_wait_that_expires_is_reported_and_every_kernel_still_ends(amd):
    """Failure path of the waits between work-groups, forced from the host: with spin_limit < 0
    every read of a row that another band finishes in the same launch gives up at once.  The
    kernels drain normally, ckpt_check_inputs reports CKPT_E_INTERNAL, and the next ordinary solve
    into the same buffers is complete again."""
    import torch
    batch = random_chain_batch(40, 3000, 3, 61, size_hi=300, time_hi=2000, overheads=True)
    L, M, B = batch.L, batch.M, batch.B
    up = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()
    uf, ub, wa, wabar = up(batch.uf), up(batch.ub), up(batch.wa), up(batch.wabar)
    opt = dict(of=up(batch.of), ob=up(batch.ob))
    cost = torch.empty(amd.ckpt_table_elems(L, M, B), dtype=torch.int32, device="cuda")
    arg = torch.empty(amd.ckpt_table_elems(L, M, B), dtype=torch.uint8, device="cuda")
    ws = torch.empty(amd.ckpt_workspace_bytes(L, M, B), dtype=torch.uint8, device="cuda")
    amd.ckpt_solve_batched_opts(uf, ub, wa, wabar, L, M, B, cost, arg, ws, spin_limit=-1, **opt)
    lib = amd.load_library()
    flags = np.zeros(B, np.int32)
    rc = lib.ckpt_check_inputs(ws.data_ptr(), L, M, B, None, flags.ctypes.data)
    torch.cuda.synchronize()
    assert rc == -9, rc
    amd.ckpt_solve_batched(uf, ub, wa, wabar, L, M, B, cost, arg, ws, **opt)
    assert amd.ckpt_check_inputs(ws, L, M, B).tolist() == [0] * B
    ref = amd.solve(batch, row_launches=1)
    pitch = amd.ckpt_row_pitch(M)
    assert (cost.view(B, -1, pitch)[:, :, :M + 1] == ref.cost[:, :, :M + 1]).all()
    assert (arg.view(B, -1, pitch)[:, :, :M + 1] == ref.arg[:, :, :M + 1]).all()


def test_solve_with_other_streams_busy(amd, oracle_mod):
    """A split solve issued while streams of the process that the library does not know are busy
    with copies and kernels of their own."""
    import torch
    batch = random_chain_batch(32, 30000, 5, 38, size_hi=1000, time_hi=5000, overheads=True)
    busy = [torch.cuda.Stream() for _ in range(3)]
    blobs = [torch.zeros(1 << 24, dtype=torch.int32, device="cuda") for _ in busy]
    for _ in range(20):
        for st, blob in zip(busy, blobs):
            with torch.cuda.stream(st):
                blob.add_(1)
                blob.copy_(blob.flip(0))
    sol = amd.solve(batch, check=False)
    for st, blob in zip(busy, blobs):
        with torch.cuda.stream(st):
            blob.add_(1)
    torch.cuda.synchronize()
    assert_tables_equal(oracle_mod, batch, sol, nthreads=8)
    assert all(int(blob[0]) == 21 for blob in blobs)


def test_capture_of_a_long_chain_on_a_split_batch(amd):
    """L >= 157 (the frontier kernel needs its enlarged on-chip allocation) on a batch large
    enough to be split, captured after ckpt_init and replayed against the eager tables."""
    import torch
    batch = random_chain_batch(160, 2500, 4, 39, size_hi=60, time_hi=3000)
    L, M, B = batch.L, batch.M, batch.B
    amd.ckpt_init()
    up = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()
    uf, ub, wa, wabar = up(batch.uf), up(batch.ub), up(batch.wa), up(batch.wabar)
    cost = torch.empty(amd.ckpt_table_elems(L, M, B), dtype=torch.int32, device="cuda")
    arg = torch.empty(amd.ckpt_table_elems(L, M, B), dtype=torch.uint8, device="cuda")
    ws = torch.empty(amd.ckpt_workspace_bytes(L, M, B), dtype=torch.uint8, device="cuda")
    eager = amd.solve(batch)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        amd.ckpt_solve_batched(uf, ub, wa, wabar, L, M, B, cost, arg, ws)
    torch.cuda.synchronize()
    pitch = amd.ckpt_row_pitch(M)
    for _ in range(2):
        cost.fill_(-5)
        arg.fill_(77)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert (cost.view(B, -1, pitch)[:, :, :M + 1] == eager.cost[:, :, :M + 1]).all()
        assert (arg.view(B, -1, pitch)[:, :, :M + 1] == eager.arg[:, :, :M + 1]).all()


def test_schedule_from_gpu_table_runs_in_budget(amd, oracle_mod):
    batch = make_config(1)
    L, M = batch.L, batch.M
    ch = batch.chain(0)
    sol = amd.solve(batch)
    arg_h = sol.arg[0].cpu().numpy()
    cost_h = sol.cost[0].cpu().numpy()
    root = amd.ckpt_row_index(L, 1, L)
    checked = 0
    for m in range(0, M + 1, 16):
        if cost_h[root, m] >= amd.CKPT_INF:
            continue
        ops = amd.ckpt_schedule(arg_h, ch[2], ch[3], L, M, 1, L, m)
        time, peak = simulate(ops, 1, L, *ch)
        assert time == cost_h[root, m] and peak <= m
        checked += 1
    assert checked > 5


def test_solve_on_a_side_stream(amd, oracle_mod):
    import torch
    batch = make_config(1)
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        sol = amd.solve(batch)
    st.synchronize()
    assert_tables_equal(oracle_mod, batch, sol)


@pytest.mark.parametrize("which", ["one_stream", "four_streams"])
def test_solve_can_be_captured_in_a_hip_graph(amd, which):
    """Capture one solve, replay it several times with eager work and synchronisations in between,
    and compare every replay with the eager tables.  The larger batch is split over the library's
    side streams, so its capture includes their fork and join."""
    import torch
    batch = make_config(2) if which == "one_stream" else \
        random_chain_batch(32, 30000, 5, 36, size_hi=1000, time_hi=5000, overheads=True)
    L, M, B = batch.L, batch.M, batch.B
    up = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()
    uf, ub, wa, wabar = up(batch.uf), up(batch.ub), up(batch.wa), up(batch.wabar)
    opt = dict(wdelta=up(batch.wdelta), of=up(batch.of), ob=up(batch.ob))
    cost = torch.empty(amd.ckpt_table_elems(L, M, B), dtype=torch.int32, device="cuda")
    arg = torch.empty(amd.ckpt_table_elems(L, M, B), dtype=torch.uint8, device="cuda")
    ws = torch.empty(amd.ckpt_workspace_bytes(L, M, B), dtype=torch.uint8, device="cuda")
    eager = amd.solve(batch)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        amd.ckpt_solve_batched(uf, ub, wa, wabar, L, M, B, cost, arg, ws, **opt)      # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        amd.ckpt_solve_batched(uf, ub, wa, wabar, L, M, B, cost, arg, ws, **opt)
    torch.cuda.synchronize()
    pitch = amd.ckpt_row_pitch(M)
    for _ in range(3):
        cost.fill_(-5)
        arg.fill_(77)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert (cost.view(B, -1, pitch)[:, :, :M + 1] == eager.cost[:, :, :M + 1]).all()
        assert (arg.view(B, -1, pitch)[:, :, :M + 1] == eager.arg[:, :, :M + 1]).all()


@pytest.mark.parametrize("which", ["small", "split"])
def test_concurrent_solves_on_two_streams(amd, oracle_mod, which):
    """Two solves in flight at once on different caller streams; the larger ones both use the
    library's side streams."""
    import torch
    if which == "small":
        b1, b2 = make_config(2), random_chain_batch(40, 300, 4, 33, size_hi=9, overheads=True)
    else:
        b1 = random_chain_batch(48, 16000, 16, 37, size_hi=600, time_hi=3000)
        b2 = random_chain_batch(32, 30000, 5, 38, size_hi=1000, time_hi=5000, overheads=True)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    with torch.cuda.stream(s1):
        sol1 = amd.solve(b1, check=False)
    with torch.cuda.stream(s2):
        sol2 = amd.solve(b2, check=False)
    torch.cuda.synchronize()
    assert_tables_equal(oracle_mod, b1, sol1, nthreads=8, chains=[0, 7, 15])
    assert_tables_equal(oracle_mod, b2, sol2, nthreads=8)


def _full_solution(amd, cfg):
    """Solve a large configuration once per test session (the launch configuration the benchmark times)."""
    import torch
    if cfg not in _full:
        _full.clear()                       # keep one multi-GB table set alive at a time
        torch.cuda.empty_cache()
        batch = make_config(cfg)
        sol = amd.solve(batch)
        torch.cuda.synchronize()
        _full[cfg] = (batch, sol)
    return _full[cfg]


@pytest.mark.parametrize("cfg,group", [(3, g) for g in range(8)] + [(4, g) for g in range(8)])
def test_configs_full_size(amd, oracle_mod, cfg, group):
    """The two large configurations: full tables of every chain (cfg 3: eight chains per case,
    cfg 4: one chain per case).  The oracle runs on all host cores."""
    batch, sol = _full_solution(amd, cfg)
    per = batch.B // 8
    chains = list(range(group * per, (group + 1) * per))
    print(f"case {batch.name} chains {chains}", flush=True)
    nthreads = min(16, oracle_mod.max_threads())
    assert_tables_equal(oracle_mod, batch, sol, nthreads=nthreads, chains=chains)


def test_cfg4_infeasible_share(amd):
    batch, sol = _full_solution(amd, 4)
    n_inf = sum(int((sol.cost[b, :, :batch.M + 1] == amd.CKPT_INF).sum()) for b in range(batch.B))
    frac = n_inf / (batch.B * amd.ckpt_table_rows(batch.L) * (batch.M + 1))
    assert abs(frac - 0.30) < 0.01, frac
    _full.clear()


def test_split_requested_inside_a_capture_without_init_is_refused():
    """Nothing is created behind a capture: a fresh process that asks for a split solve while its
    stream is being captured, without ckpt_init, gets CKPT_E_NOTREADY and a capture that still
    ends normally; after ckpt_init the same capture succeeds.  Runs in a process of its own
    because the helper streams of this one may exist already."""
    import os
    import subprocess
    import sys
    code = r'''
import numpy as np, torch, sys
sys.path.insert(0, %r)
import paper_2302_02599_amd as amd
from workloads import make_config
batch = make_config(2)
L, M, B = batch.L, batch.M, batch.B
up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
uf, ub, wa, wabar = up(batch.uf), up(batch.ub), up(batch.wa), up(batch.wabar)
cost = torch.empty(amd.ckpt_table_elems(L, M, B), dtype=torch.int32, device="cuda")
arg = torch.empty(amd.ckpt_table_elems(L, M, B), dtype=torch.uint8, device="cuda")
ws = torch.empty(amd.ckpt_workspace_bytes(L, M, B), dtype=torch.uint8, device="cuda")
side = torch.cuda.Stream()
torch.cuda.synchronize()
codes = []
for attempt in range(2):
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        try:
            amd.ckpt_solve_batched_opts(uf, ub, wa, wabar, L, M, B, cost, arg, ws, groups=2)
            codes.append(0)
        except amd.CkptError as e:
            codes.append(e.code)
    torch.cuda.synchronize()
    if attempt == 0:
        amd.ckpt_init()
graph.replay()
torch.cuda.synchronize()
ref = amd.solve(batch, groups=1)
ok = bool((cost.view(B, -1, amd.ckpt_row_pitch(M))[:, :, :M + 1] == ref.cost[:, :, :M + 1]).all())
print("RESULT", codes, ok)
''' % os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    out = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300)
    assert "RESULT [-8, 0] True" in out.stdout, out.stdout[-2000:] + out.stderr[-2000:]
