"""Host sanitizer job: the CPU oracle (oracle/ckpt_oracle.c) and the host-only sources of the
library (table layout, budget list, schedule walk, block indices, linearisation) are compiled
with -fsanitize=address,undefined into one driver (tests/sanitize_host_driver.cpp) and run on
the inputs of the host tests; the driver's results must equal those of the ordinary builds, and
any sanitizer report (heap overflow, signed overflow, misaligned or out-of-range access)
aborts it.  CPU only."""
import os
import random
import subprocess

import numpy as np
import pytest

from workloads import make_config, random_chain_batch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2302_02599_amd", "csrc")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-g", "-O1", "-fopenmp"]


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    out = tmp_path_factory.mktemp("sanitize")
    obj = str(out / "oracle.o")
    subprocess.check_call(["gcc", *SAN, "-Wall", "-Wextra", "-c", os.path.join(ROOT, "oracle", "ckpt_oracle.c"), "-o", obj])
    exe = str(out / "driver")
    subprocess.check_call(["g++", *SAN, "-std=c++17", "-Wall", "-I", os.path.join(ROOT, "include"),
                           os.path.join(ROOT, "tests", "sanitize_host_driver.cpp"), obj,
                           os.path.join(CSRC, "ckpt_host.cpp"), os.path.join(CSRC, "ckpt_schedule.cpp"),
                           os.path.join(CSRC, "ckpt_linearize.cpp"), "-o", exe])

    def run(script):
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
                   OMP_NUM_THREADS="2")
        r = subprocess.run([exe], input=script, capture_output=True, text=True, timeout=600, env=env)
        assert r.returncode == 0, r.stderr[-4000:]
        assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]
        return r.stdout.splitlines()
    run.dir = out
    return run


@pytest.fixture(scope="module")
def amd():
    import paper_2302_02599_amd as amd
    if not os.path.exists(amd.lib_path()):
        from paper_2302_02599_amd.build import build_library
        build_library()
    amd.load_library()
    return amd


def _chain_cmd(L, M, ch):
    return f"chain {L} {M} " + " ".join(" ".join(str(int(v)) for v in a) for a in ch) + "\n"


def _ops_text(ops):
    return "".join(f" {k}:{s}" for k, s in ops)


@pytest.mark.parametrize("which", ["cfg0", "cfg1", "rand_all_arrays", "saturating", "outside_model"])
def test_oracle_and_schedule_walk_under_sanitizers(driver, amd, oracle_mod, which):
    if which == "cfg0":
        batch = make_config(0)
    elif which == "cfg1":
        batch = make_config(1)
        batch.M = 160
    else:
        batch = random_chain_batch(11, 70, 1, 88, size_hi=7, overheads=True, own_wdelta=True, zero_sizes=True)
        if which == "saturating":
            batch.uf[:] = 150_000_000
            batch.ub[:] = 300_000_000
        if which == "outside_model":
            batch.wabar[0, ::2] = 0
    L, M = batch.L, batch.M
    ch = batch.chain(0)
    cost, choice = oracle_mod.solve_chain(L, M, *ch)
    pc, pk = driver.dir / f"{which}.cost", driver.dir / f"{which}.choice"
    script = _chain_cmd(L, M, ch) + f"dump {pc} {pk}\n"
    cells = [(s, t) for s in range(1, L + 1) for t in range(s, L + 1)]
    for s, t in cells:
        script += f"thresholds {s} {t}\n"
    rng = random.Random(3)
    walks = [(1, L, m) for m in range(0, M + 1, max(1, M // 25))] + [(1, L, M + 7)] + \
            [(s, t, rng.randrange(M + 1)) for s, t in rng.sample(cells, min(len(cells), 25))]
    cap = L * (L + 1) // 2 + L
    for s, t, m in walks:
        script += f"schedule {s} {t} {m} {cap}\n"
    script += f"schedule 1 {L} {M} 3\nschedule 1 {L} -1 {cap}\nschedule 2 1 {M} {cap}\n"
    out = driver(script)
    assert out[0] == "chain 0" and out[1] == f"dump {L * L * (M + 1)}"
    got_cost = np.fromfile(pc, np.int32).reshape(L, L, M + 1)
    got_choice = np.fromfile(pk, np.int16).reshape(L, L, M + 1)
    iu = np.triu_indices(L)
    assert (got_cost[iu] == cost[iu]).all() and (got_choice[iu] == choice[iu]).all()
    line = 2
    for s, t in cells:
        want = oracle_mod.thresholds(L, ch[2], ch[3], ch[4], ch[5], ch[6], s, t)
        assert out[line] == f"thresholds {want[0]} {want[1]}", (s, t)
        line += 1
    feasible = 0
    for s, t, m in walks:
        mm = min(m, M)
        if cost[s - 1, t - 1, mm] >= oracle_mod.INF:
            assert out[line] == "schedule -3", (s, t, m)
            line += 1
            continue
        ops = oracle_mod.reconstruct(choice, ch[2], ch[3], s, t, mm)
        assert out[line] == f"schedule {len(ops)}" + _ops_text(ops), (s, t, m)
        line += 1
        feasible += 1
        if s == 1 and t == L:
            blocks, n = oracle_mod.block_indices(ops, L)
            assert out[line] == f"blocks {n}" + "".join(f" {b}" for b in blocks), m
            line += 1
    assert feasible > 5
    assert out[line:line + 3] == ["schedule -4" if cost[0, L - 1, M] < oracle_mod.INF else "schedule -3",
                                  "schedule -1", "schedule -1"]


def test_block_indices_of_bad_lists_under_sanitizers(driver):
    out = driver("blocks 3 8 1:1 2:2 0:3 3:3 0:1 0:2 3:2 3:1\n"      # C1 N2 A3 ...
                 "blocks 3 2 0:1 3:1\n"                                # shorter than the chain
                 "blocks 2 3 2:1 0:2 3:2\n"                            # F_null^1
                 "blocks 2 3 0:1 3:2 3:2\n"
                 "blocks 254 0\n")
    assert out == ["blocks 1 0 0 -1", "blocks -7", "blocks -7", "blocks -7", "blocks -7"]


def test_linearize_under_sanitizers(driver, oracle_mod):
    P, SEED, NOND, INPL, COMM = 1, 2, 4, 8, 16
    script, want = "", []
    for seed in range(20):
        rng = random.Random(100 + seed)
        n = rng.randrange(1, 60)
        children = [[] for _ in range(n)]
        for v in range(1, n):
            for u in {rng.randrange(max(0, v - 6), v) for _ in range(rng.choice([1, 1, 2, 3]))}:
                children[u].append(v)
        flags = []
        for v in range(n):
            if not any(v in children[u] for u in range(n)):
                flags.append(P | (SEED if rng.random() < 0.4 else 0))
            elif not children[v]:
                flags.append(P)
            else:
                r = rng.random()
                flags.append(NOND if r < 0.1 else INPL if r < 0.2 else COMM if r < 0.27 else 0)
        script += f"linearize {n} " + " ".join(f"{len(c)} " + " ".join(map(str, c)) for c in children) + " " + \
                  " ".join(map(str, flags)) + "\n"
        group, common, ngroups = oracle_mod.linearize(children, flags)
        want.append(f"linearize {ngroups} groups " + " ".join(map(str, group)) + " common " +
                    " ".join(str(int(c)) for c in common))
    script += "linearize 0\nlinearize 2 1 0 0 0 0\n"          # empty graph; an edge that is not forward
    want += ["linearize 0 groups common", "linearize -1 groups common"]
    assert driver(script) == want


def test_layout_and_budget_sweep_under_sanitizers(driver, amd, oracle_mod):
    cases = [(1000, 1, 10, 10), (1, 1, 1, 16), (2 ** 62, 1, 3, 2), (2 ** 62, 1, 1, 3), (7, 0, 5, 4),
             (123456789012, 37, 100, 16), (5, 2 ** 31 - 1, 1, 16), (0, 1, 10, 3), (5, 1, 10, 17)]
    out = driver("".join(f"sweep {b} {n} {d} {c}\n" for b, n, d, c in cases) + "layout 7 130\nlayout 254 65535\n")
    lib = amd.load_library()
    for (b, n, d, c), line in zip(cases, out):
        try:
            want = "sweep 0 " + " ".join(map(str, amd.ckpt_budget_sweep(b, n, d, c)))
            assert amd.ckpt_budget_sweep(b, n, d, c) == oracle_mod.budget_sweep(b, n, d, c)
        except amd.CkptError as e:
            want = f"sweep {e.code}"
        assert line == want, (b, n, d, c)
    for (L, M), line in zip([(7, 130), (254, 65535)], out[len(cases):]):
        want = f"layout {amd.ckpt_row_pitch(M)} {amd.ckpt_table_rows(L)} {amd.ckpt_table_elems(L, M, 3)}"
        want += "".join(f" {amd.ckpt_row_index(L, s, t)}" for s in range(L + 2) for t in range(L + 2))
        assert line == want + " " + lib.ckpt_strerror(-7).decode()
