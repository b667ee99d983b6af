"""The benchmark's work and byte models against direct enumeration on small chains.

bench.py prices its figures with closed forms (cells, candidates) and with per-kernel models
(which candidates the blocked kernels handle, how many operand loads a row costs); a wrong
model would misstate throughput and roofline, so each is recounted here the slow way.
"""
import pytest

import bench


@pytest.mark.parametrize("L", [1, 2, 7, 8, 9, 23, 40])
def test_cells_and_candidates(L):
    M, B = 5, 3
    cells = sum(1 for s in range(1, L + 1) for t in range(s, L + 1))
    # one candidate per cell for C_all (the only one when s == t) and one per s' in s+1..t
    evals = sum(1 + (t - s) for s in range(1, L + 1) for t in range(s, L + 1))
    assert bench.counts(L, M, B) == (cells * (M + 1) * B, evals * (M + 1) * B)


def classify(L, T):
    """For every checkpoint split (i, j, q), 0-based, q in i+1..j: which kernel evaluates it."""
    middle = near_i = near_j = 0
    middle_cells = set()
    for i in range(L):
        for j in range(i + 1, L):
            I, J = i // T, j // T
            for q in range(i + 1, j + 1):
                if J - I >= 2 and (I + 1) * T <= q <= J * T:
                    middle += 1
                elif q < (I + 1) * T or (J - I == 1 and q == J * T):
                    near_i += 1       # right operand is a lower row of the same tile
                else:
                    near_j += 1       # left operand is an earlier cell of the same row
            if J - I >= 2:
                middle_cells.add((i, j))
    return middle, near_i, near_j, len(middle_cells)


@pytest.mark.parametrize("L", [8, 16, 17, 24, 31, 48])
def test_gemm_work_is_the_middle_splits(L):
    T, M, B = 8, 3, 2
    middle, near_i, near_j, cells = classify(L, T)
    assert middle + near_i + near_j == sum(j - i for i in range(L) for j in range(i, L))
    got_evals, got_cells, _ = bench.gemm_work(L, M, B, T)
    # rows of a tile always number T, columns only those that exist in a ragged last block
    assert got_evals == middle * (M + 1) * B
    assert got_cells == cells * (M + 1) * B


def loads_of_row(L, T, i, J):
    """Operand loads of a lane that finishes row i in column block J, counted split by split:
    9 per split in the row block (D = 1: and the first stage of the column block), 1 per split
    in the column block, 1 C_all operand per cell with j > i.  Full blocks only."""
    I, D = i // T, J - i // T
    cols = [j for j in range(J * T, J * T + T) if j >= i]
    loads = 0
    if D >= 1:
        loads += (len(range(i + 1, (I + 1) * T)) + (1 if D == 1 else 0)) * (1 + T)
    for j in cols:
        loads += sum(1 for q in range(i + 1, j + 1) if q > J * T or D == 0)
        loads += 1 if j > i else 0
    return loads, len(cols)


@pytest.mark.parametrize("L", [8, 16, 24, 40])
def test_bytes_count_every_operand_once(L):
    """Rows of all tiles but row 7 of the tiles of D >= 2 belong to row_kernel (4 B per load,
    5 B of partial per cell of a D >= 2 tile, 5 B stored per cell); row 7 of those tiles belongs
    to gemm_kernel, next to 1 B per middle candidate and 5 B stored per cell of the tile."""
    T, M, B = 8, 0, 1
    row_total = gemm_loads = 0
    for i in range(L):
        for J in range(i // T, L // T):
            D = J - i // T
            loads, stored = loads_of_row(L, T, i, J)
            if D >= 2 and i % T == T - 1:
                gemm_loads += loads
            else:
                row_total += 4 * loads + (5 * T if D >= 2 else 0) + 5 * stored
    assert bench.row_bytes(L, M, B, T) == row_total
    middle, _, _, cells = classify(L, T)
    assert bench.gemm_work(L, M, B, T) == (middle, cells, gemm_loads)
    assert bench.gemm_bytes(L, M, B, T) == middle + 5 * cells + 4 * gemm_loads
