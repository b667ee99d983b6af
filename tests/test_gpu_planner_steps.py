"""GPU parity of the planner-side steps: plan selection, discretisation, batched schedule walk.
Integer work: exact equality with the oracle."""
import numpy as np
import pytest

from workloads import ChainBatch, make_config

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def amd():
    import torch
    assert torch.cuda.is_available()
    import paper_2302_02599_amd as amd
    amd.load_library()
    return amd


@pytest.fixture(scope="module")
def solved(amd, oracle_mod):
    batch = make_config(2)
    sol = amd.solve(batch)
    tables = oracle_mod.solve_batch(batch, nthreads=8)
    return batch, sol, tables


def _budget_sets(batch, tables, oracle_mod):
    L, M, B = batch.L, batch.M, batch.B
    rng = np.random.default_rng(5)
    first = [int(np.argmax(t[0][0, L - 1] < oracle_mod.INF)) for t in tables]
    yield "full", [M] * B
    yield "random", rng.integers(0, M, B, endpoint=True).tolist()
    yield "none_feasible", [f - 1 for f in first]
    yield "one_feasible", [f - 1 for f in first[:-1]] + [first[-1]]
    yield "mixed_signs_and_overshoot", [(-1 if b % 3 == 0 else M + 50 * b) for b in range(B)]


def test_select_plan(amd, oracle_mod, solved):
    import torch
    batch, sol, tables = solved
    L, M, B = batch.L, batch.M, batch.B
    for name, budgets in _budget_sets(batch, tables, oracle_mod):
        out = torch.full((2,), -7, dtype=torch.int32, device="cuda")
        amd.ckpt_select_plan(sol.cost, L, M, B, torch.tensor(budgets, dtype=torch.int32, device="cuda"), out)
        want = oracle_mod.select_plan([t[0] for t in tables], L, budgets)
        assert tuple(out.cpu().tolist()) == want, name


def test_select_plan_many_chains_and_ties(amd, oracle_mod):
    """More chains than threads of the selection block, with duplicated chains (ties)."""
    import torch
    base = make_config(1)
    B = 600
    reps = lambda a: np.repeat(a, B, axis=0)
    batch = ChainBatch("ties", base.L, 160, B, reps(base.uf), reps(base.ub), reps(base.wa), reps(base.wabar))
    batch.uf = batch.uf.copy()
    batch.uf[:300, 0] += 3           # the first half is slower: the winner is chain 300, not 0
    sol = amd.solve(batch)
    budgets = [160] * B
    out = torch.zeros(2, dtype=torch.int32, device="cuda")
    amd.ckpt_select_plan(sol.cost, batch.L, batch.M, B, torch.tensor(budgets, dtype=torch.int32, device="cuda"), out)
    t_slow = oracle_mod.solve_chain(batch.L, batch.M, *batch.chain(0))[0]
    t_fast = oracle_mod.solve_chain(batch.L, batch.M, *batch.chain(300))[0]
    want = oracle_mod.select_plan([t_slow] * 300 + [t_fast] * 300, batch.L, budgets)
    assert want[0] == 300 and tuple(out.cpu().tolist()) == want


@pytest.mark.parametrize("L,M,B,seed", [(1, 1, 1, 0), (7, 64, 3, 1), (48, 1024, 16, 2), (192, 4096, 8, 3), (33, 1 << 20, 2, 4)])
def test_discretize(amd, oracle_mod, L, M, B, seed):
    import torch
    rng = np.random.default_rng(seed)
    big = 1 << 41
    arrays = {"wa": rng.integers(0, big, (B, L + 1)), "wabar": rng.integers(0, big, (B, L)),
              "wdelta": rng.integers(0, 1 << 20, (B, L + 1)), "of": rng.integers(0, 3, (B, L)),
              "ob": rng.integers(0, big, (B, L))}
    budget = rng.integers(1, 1 << 40, B)
    if B > 1:
        budget[-1] = 1                                 # huge quotients: clamps
    arrays["wa"][0, 0] = 0
    arrays["wabar"][0, 0] = int(budget[0])            # exactly the whole budget -> M slots
    dev = {k: torch.from_numpy(v.astype(np.int64)).cuda() for k, v in arrays.items()}
    outs = {k: torch.full(v.shape, -1, dtype=torch.int32, device="cuda") for k, v in arrays.items()}
    amd.ckpt_discretize(dev["wa"], dev["wabar"], torch.from_numpy(budget.astype(np.int64)).cuda(), L, M, B,
                        outs["wa"], outs["wabar"], bytes_wdelta=dev["wdelta"], bytes_of=dev["of"], bytes_ob=dev["ob"],
                        wdelta=outs["wdelta"], of=outs["of"], ob=outs["ob"])
    for k, v in arrays.items():
        got = outs[k].cpu().numpy()
        for b in range(B):
            assert got[b].tolist() == oracle_mod.discretize(v[b].tolist(), int(budget[b]), M), (k, b)
    assert outs["wabar"][0, 0].item() == M


def test_discretize_optional_arrays_left_alone(amd):
    import torch
    L, M, B = 5, 16, 2
    z = lambda n: torch.ones((B, n), dtype=torch.int64, device="cuda")
    wa = torch.full((B, L + 1), -1, dtype=torch.int32, device="cuda")
    wabar = torch.full((B, L), -1, dtype=torch.int32, device="cuda")
    amd.ckpt_discretize(z(L + 1), z(L), torch.full((B,), 16, dtype=torch.int64, device="cuda"), L, M, B, wa, wabar)
    assert (wa == 1).all() and (wabar == 1).all()


def test_schedule_batched_matches_host_walk_and_oracle(amd, oracle_mod, solved):
    import torch
    batch, sol, tables = solved
    L, M, B = batch.L, batch.M, batch.B
    cap = L * (L + 1) // 2 + L
    wa = torch.from_numpy(batch.wa).cuda()
    wabar = torch.from_numpy(batch.wabar).cuda()
    ws = torch.empty(amd.ckpt_schedule_workspace_bytes(L, B), dtype=torch.uint8, device="cuda")
    arg_host = sol.arg.cpu().numpy()
    for name, budgets in _budget_sets(batch, tables, oracle_mod):
        ops = torch.zeros((B, cap, 2), dtype=torch.uint8, device="cuda")
        n_ops = torch.zeros(B, dtype=torch.int32, device="cuda")
        amd.ckpt_schedule_batched(sol.arg, wa, wabar, L, M, B, torch.tensor(budgets, dtype=torch.int32, device="cuda"),
                                  ops, cap, n_ops, ws)
        ops_h, n_h = ops.cpu().numpy(), n_ops.cpu().numpy()
        for b in range(B):
            m = budgets[b]
            if m < 0:
                assert n_h[b] == -1, (name, b)
                continue
            m = min(m, M)
            if tables[b][0][0, L - 1, m] >= oracle_mod.INF:
                assert n_h[b] == -3, (name, b)
                continue
            want = oracle_mod.reconstruct(tables[b][1], batch.wa[b], batch.wabar[b], 1, L, m)
            got = [tuple(x) for x in ops_h[b, :n_h[b]].tolist()]
            assert got == want, (name, b)
            assert got == amd.ckpt_schedule(arg_host[b], batch.wa[b], batch.wabar[b], L, M, 1, L, m), (name, b)


def test_schedule_batched_small_capacity_and_corrupt_table(amd, solved):
    import torch
    batch, sol, _ = solved
    L, M, B = batch.L, batch.M, batch.B
    wa = torch.from_numpy(batch.wa).cuda()
    wabar = torch.from_numpy(batch.wabar).cuda()
    ws = torch.empty(amd.ckpt_schedule_workspace_bytes(L, B), dtype=torch.uint8, device="cuda")
    budgets = torch.full((B,), M, dtype=torch.int32, device="cuda")
    ops = torch.zeros((B, 5, 2), dtype=torch.uint8, device="cuda")
    n_ops = torch.zeros(B, dtype=torch.int32, device="cuda")
    amd.ckpt_schedule_batched(sol.arg, wa, wabar, L, M, B, budgets, ops, 5, n_ops, ws)
    assert (n_ops == -4).all()
    broken = sol.arg.clone()
    broken[3, amd.ckpt_row_index(L, 1, L), M] = L + 9
    cap = L * (L + 1) // 2 + L
    ops = torch.zeros((B, cap, 2), dtype=torch.uint8, device="cuda")
    amd.ckpt_schedule_batched(broken, wa, wabar, L, M, B, budgets, ops, cap, n_ops, ws)
    got = n_ops.cpu().tolist()
    assert got[3] == -7 and all(v > 0 for k, v in enumerate(got) if k != 3)


def _walk_on_device(amd, batch, sol, budgets):
    import torch
    L, M, B = batch.L, batch.M, batch.B
    cap = L * (L + 1) // 2 + L
    ws = torch.empty(amd.ckpt_schedule_workspace_bytes(L, B), dtype=torch.uint8, device="cuda")
    ops = torch.zeros((B, cap, 2), dtype=torch.uint8, device="cuda")
    n_ops = torch.zeros(B, dtype=torch.int32, device="cuda")
    amd.ckpt_schedule_batched(sol.arg, torch.from_numpy(batch.wa).cuda(), torch.from_numpy(batch.wabar).cuda(), L, M, B,
                              torch.tensor(budgets, dtype=torch.int32, device="cuda"), ops, cap, n_ops, ws)
    return ops, cap, n_ops


def _check_block_indices(amd, oracle_mod, batch, sol, budgets, name):
    """Device block indices of every chain against the oracle's, computed from the oracle-checked
    operation list of the same chain."""
    import torch
    L, B = batch.L, batch.B
    ops, cap, n_ops = _walk_on_device(amd, batch, sol, budgets)
    blocks = torch.full((B, L), -9, dtype=torch.int32, device="cuda")
    n_blocks = torch.full((B,), -9, dtype=torch.int32, device="cuda")
    amd.ckpt_block_indices_batched(ops, cap, n_ops, L, B, blocks, n_blocks)
    ops_h, n_h, blocks_h, nb_h = ops.cpu().numpy(), n_ops.cpu().tolist(), blocks.cpu().tolist(), n_blocks.cpu().tolist()
    shapes = set()
    for b in range(B):
        if n_h[b] < 0:
            assert nb_h[b] == n_h[b] and blocks_h[b] == [-1] * L, (name, b)
            continue
        want, want_n = oracle_mod.block_indices([tuple(x) for x in ops_h[b, :n_h[b]].tolist()], L)
        assert (blocks_h[b], nb_h[b]) == (want, want_n), (name, b)
        shapes.add(tuple(want))
    return shapes


def test_block_indices_batched(amd, oracle_mod, solved):
    batch, sol, tables = solved
    shapes = set()
    for name, budgets in _budget_sets(batch, tables, oracle_mod):
        shapes |= _check_block_indices(amd, oracle_mod, batch, sol, budgets, name)
    assert len(shapes) > 4


def test_block_indices_batched_many_chains_and_long_chains(amd, oracle_mod):
    """700 chains (more than any block has threads), and chains longer than one pass of 64 stages
    with tight budgets so that blocks straddle the passes."""
    from workloads.chains import random_chain_batch
    rng = np.random.default_rng(11)
    batch = random_chain_batch(10, 100, 700, 34, size_hi=9)
    sol = amd.solve(batch)
    shapes = _check_block_indices(amd, oracle_mod, batch, sol, rng.integers(-1, 101, 700).tolist(), "many")
    assert len(shapes) > 20
    batch = random_chain_batch(150, 400, 3, 42, size_hi=9, time_hi=900)
    sol = amd.solve(batch)
    cost_h = sol.cost[:, amd.ckpt_row_index(150, 1, 150), :401].cpu().numpy()
    first = [int(np.argmax(cost_h[b] < amd.CKPT_INF)) for b in range(3)]
    for name, budgets in (("tightest", first), ("tight", [f + 9 for f in first]), ("roomy", [400] * 3)):
        shapes = _check_block_indices(amd, oracle_mod, batch, sol, budgets, name)
        if name == "tightest":
            assert any(max(sh) >= 1 and sum(1 for v in sh if v >= 0) > 64 for sh in shapes)


def test_block_indices_batched_rejects_edited_lists(amd, solved):
    import torch
    batch, sol, _ = solved
    L, M, B = batch.L, batch.M, batch.B
    ops, cap, n_ops = _walk_on_device(amd, batch, sol, [M] * B)
    ops_h = ops.cpu().numpy().copy()
    ops_h[1, 0] = (2, 1)                  # chain 1: F_null^1 has no block to continue
    ops_h[2, 5, 1] = 9                    # chain 2: stage out of order in the first sweep
    ops_h[3, L] = (0, L)                  # chain 3: no B^L after the first sweep
    n_h = n_ops.cpu().numpy().copy()
    n_h[4] = L                            # chain 4: list shorter than the chain
    n_h[5] = cap + 1                      # chain 5: longer than the buffer
    n_h[6] = -3                           # chain 6: the walk had failed
    blocks = torch.full((B, L), -9, dtype=torch.int32, device="cuda")
    n_blocks = torch.full((B,), -9, dtype=torch.int32, device="cuda")
    amd.ckpt_block_indices_batched(torch.from_numpy(ops_h).cuda(), cap, torch.from_numpy(n_h).cuda(), L, B, blocks,
                                   n_blocks)
    got = n_blocks.cpu().tolist()
    assert got[1:7] == [-7, -7, -7, -7, -1, -3] and got[0] >= 0 and got[7] >= 0
    assert (blocks[1:7] == -1).all()


def _simulate_on_device(amd, batch, ops, cap, n_ops):
    import torch
    up = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()
    B = batch.B
    time = torch.full((B,), -9, dtype=torch.int64, device="cuda")
    peak = torch.full((B,), -9, dtype=torch.int64, device="cuda")
    status = torch.full((B,), -9, dtype=torch.int32, device="cuda")
    amd.ckpt_simulate_batched(up(batch.uf), up(batch.ub), up(batch.wa), up(batch.wabar), batch.L, B, ops, cap, n_ops,
                              time, peak, status, wdelta=up(batch.wdelta), of=up(batch.of), ob=up(batch.ob))
    return time.cpu().tolist(), peak.cpu().tolist(), status.cpu().tolist()


def _oracle_simulation(oracle_mod, batch, b, ops):
    try:
        return oracle_mod.simulate(ops, batch.L, *batch.chain(b)) + (0,)
    except ValueError:
        return (-1, -1, -7)


def _check_walk_then_simulate(amd, oracle_mod, batch, sol, tables, budgets, name):
    import torch
    L, M, B = batch.L, batch.M, batch.B
    cap = L * (L + 1) // 2 + L
    ws = torch.empty(amd.ckpt_schedule_workspace_bytes(L, B), dtype=torch.uint8, device="cuda")
    ops = torch.zeros((B, cap, 2), dtype=torch.uint8, device="cuda")
    n_ops = torch.zeros(B, dtype=torch.int32, device="cuda")
    amd.ckpt_schedule_batched(sol.arg, torch.from_numpy(batch.wa).cuda(), torch.from_numpy(batch.wabar).cuda(), L, M, B,
                              torch.tensor(budgets, dtype=torch.int32, device="cuda"), ops, cap, n_ops, ws)
    time, peak, status = _simulate_on_device(amd, batch, ops, cap, n_ops)
    n_h = n_ops.cpu().tolist()
    longest = 0
    for b in range(B):
        if n_h[b] < 0:
            assert (time[b], peak[b], status[b]) == (-1, -1, n_h[b]), (name, b)
            continue
        m = min(budgets[b], M)
        want_ops = oracle_mod.reconstruct(tables[b][1], batch.wa[b], batch.wabar[b], 1, L, m)
        want = _oracle_simulation(oracle_mod, batch, b, want_ops)
        assert (time[b], peak[b], status[b]) == want, (name, b)
        assert status[b] == 0 and time[b] == tables[b][0][0, L - 1, m] and peak[b] <= m, (name, b)
        longest = max(longest, n_h[b])
    return longest


def test_simulate_batched_confirms_the_walked_schedules(amd, oracle_mod, solved):
    batch, sol, tables = solved
    for name, budgets in _budget_sets(batch, tables, oracle_mod):
        _check_walk_then_simulate(amd, oracle_mod, batch, sol, tables, budgets, name)


def test_simulate_batched_with_overheads_own_gradient_sizes_and_long_lists(amd, oracle_mod):
    from workloads.chains import random_chain_batch
    batch = random_chain_batch(70, 700, 3, 41, size_hi=9, time_hi=900, overheads=True, own_wdelta=True)
    sol = amd.solve(batch)
    tables = oracle_mod.solve_batch(batch, nthreads=8)
    L, M = batch.L, batch.M
    first = [int(np.argmax(t[0][0, L - 1] < oracle_mod.INF)) for t in tables]
    assert all(tables[b][0][0, L - 1, first[b]] < oracle_mod.INF for b in range(batch.B))
    longest = 0
    for name, budgets in (("tightest", first), ("roomy", [M] * batch.B), ("between", [(f + M) // 3 for f in first])):
        longest = max(longest, _check_walk_then_simulate(amd, oracle_mod, batch, sol, tables, budgets, name))
    assert longest > 2 * 256  # the list is staged through on-chip memory in several parts


def test_simulate_batched_edited_lists(amd, oracle_mod):
    """Persistent schedules with random edits, most of them no longer executable, plus unknown
    operations and stages: the status, and the figures of those that still run, match the oracle."""
    import torch
    import persistent_bruteforce as bf
    from workloads.chains import random_chain_batch
    L, B, cap = 4, 256, 16
    batch = random_chain_batch(L, 8, B, 78, size_hi=6, time_hi=40, overheads=True, own_wdelta=True)
    rng = np.random.default_rng(6)
    base = [bf.flatten(t) for t in bf.trees(1, L)]
    lists = []
    for b in range(B):
        ops = list(base[int(rng.integers(len(base)))])
        for _ in range(int(rng.integers(0, 3))):
            i = int(rng.integers(len(ops)))
            edit = int(rng.integers(6))
            if edit == 0 and len(ops) > 1:
                del ops[i]
            elif edit == 1:
                ops.insert(i, ops[i])
            elif edit == 2:
                ops.insert(int(rng.integers(len(ops))), ops.pop(i))
            elif edit == 3:
                ops[i] = (int(rng.integers(0, 6)), ops[i][1])
            elif edit == 4:
                ops[i] = (ops[i][0], int(rng.integers(0, L + 3)))
            else:
                ops[i] = (ops[i][0], 255)
        lists.append(ops[:cap])
    lists[0] = []            # an empty list ends without the gradient of the input
    ops_h = np.zeros((B, cap, 2), np.uint8)
    for b, ops in enumerate(lists):
        ops_h[b, :len(ops)] = np.array(ops, np.uint8).reshape(-1, 2)
    n_h = np.array([len(o) for o in lists], np.int32)
    n_h[1], n_h[2] = cap + 1, -3          # too long for the buffer; a chain the walk gave up on
    time, peak, status = _simulate_on_device(amd, batch, torch.from_numpy(ops_h).cuda(), cap, torch.from_numpy(n_h).cuda())
    kinds = set()
    for b in range(B):
        if b == 1:
            want = (-1, -1, -1)
        elif b == 2:
            want = (-1, -1, -3)
        else:
            want = _oracle_simulation(oracle_mod, batch, b, lists[b])
        assert (time[b], peak[b], status[b]) == want, (b, lists[b])
        kinds.add(status[b])
    assert kinds == {0, -1, -3, -7}


@pytest.mark.parametrize("L,M,count,base,num,den,seed", [
    (1, 1, 1, 5, 0, 1, 0), (7, 64, 10, 1000, 1, 10, 1), (48, 1024, 10, 80 << 30, 1, 10, 2),
    (192, 4096, 16, 1 << 33, 1, 8, 3), (33, 1 << 20, 5, 12345678901, 3, 20, 4),
])
def test_discretize_sweep(amd, oracle_mod, L, M, count, base, num, den, seed):
    """One profile under every budget of the sweep: each output chain equals the oracle's
    discretisation of the profile under that budget, and the budgets equal the oracle's."""
    import torch
    rng = np.random.default_rng(seed)
    big = min(1 << 41, 4 * base)
    profile = {"wa": rng.integers(0, big, L + 1), "wabar": rng.integers(0, big, L),
               "wdelta": rng.integers(0, 1 << 20, L + 1), "of": rng.integers(0, 3, L), "ob": rng.integers(0, big, L)}
    profile["wabar"][0] = base                       # exactly the first budget -> M slots in chain 0
    dev = {k: torch.from_numpy(v.astype(np.int64)).cuda() for k, v in profile.items()}
    outs = {k: torch.full((count,) + v.shape, -1, dtype=torch.int32, device="cuda") for k, v in profile.items()}
    budgets = torch.full((count,), -1, dtype=torch.int64, device="cuda")
    amd.ckpt_discretize_sweep(dev["wa"], dev["wabar"], base, num, den, count, L, M, outs["wa"], outs["wabar"],
                              bytes_wdelta=dev["wdelta"], bytes_of=dev["of"], bytes_ob=dev["ob"],
                              wdelta=outs["wdelta"], of=outs["of"], ob=outs["ob"], budgets_out=budgets)
    assert budgets.cpu().tolist() == oracle_mod.budget_sweep(base, num, den, count)
    for k, v in profile.items():
        assert outs[k].cpu().numpy().tolist() == oracle_mod.discretize_sweep(v.tolist(), base, num, den, count, M), k
    assert outs["wabar"][0, 0].item() == M


def test_discretize_sweep_feeds_the_solver(amd, oracle_mod):
    """The sweep's output is a batch as ckpt_solve_batched takes it: tables equal the oracle's on
    the oracle's own discretisation of the same profile."""
    import torch
    L, M, count = 12, 200, 6
    rng = np.random.default_rng(9)
    by_wa, by_wabar = rng.integers(1 << 20, 1 << 24, L + 1), rng.integers(1 << 24, 1 << 26, L)
    base = 300 << 20
    wa = torch.empty((count, L + 1), dtype=torch.int32, device="cuda")
    wabar = torch.empty((count, L), dtype=torch.int32, device="cuda")
    amd.ckpt_discretize_sweep(torch.from_numpy(by_wa).cuda(), torch.from_numpy(by_wabar).cuda(), base, 1, 4, count,
                              L, M, wa, wabar)
    uf = rng.integers(1, 1000, (count, L)).astype(np.int32)
    ub = (2 * uf + rng.integers(0, 100, (count, L))).astype(np.int32)
    batch = ChainBatch("sweep", L, M, count, uf, ub, wa.cpu().numpy(), wabar.cpu().numpy())
    sol = amd.solve(batch)
    want_wa = oracle_mod.discretize_sweep(by_wa.tolist(), base, 1, 4, count, M)
    want_wabar = oracle_mod.discretize_sweep(by_wabar.tolist(), base, 1, 4, count, M)
    iu = np.triu_indices(L)
    feasible = 0
    for b in range(count):
        cost, choice = oracle_mod.solve_chain(L, M, uf[b], ub[b], want_wa[b], want_wabar[b])
        assert (sol.cost[b, :, :M + 1].cpu().numpy() == cost[iu]).all()
        assert (sol.arg[b, :, :M + 1].cpu().numpy() == choice[iu]).all()
        feasible += int(cost[0, L - 1, M] < oracle_mod.INF)
    assert 0 < feasible  # the larger budgets of the sweep make the whole chain fit
