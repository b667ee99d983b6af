"""The benchmark's work and byte models against direct enumeration on small chains.

bench.py prices its figures with closed forms (cells, candidates, the candidates that the
block-product kernel handles); a wrong model would misstate throughput and roofline, so each
is recounted here the slow way.  Bytes are not modelled any more: the kernels count them.
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
def test_gemm_evals_are_the_middle_splits(L):
    T, M, B = 8, 3, 2
    middle, near_i, near_j, _ = classify(L, T)
    assert middle + near_i + near_j == sum(j - i for i in range(L) for j in range(i, L))
    assert bench.gemm_evals(L, M, B, T) == middle * (M + 1) * B


def test_method_floor_constants():
    """5 bytes per cell (int32 cost + uint8 candidate), one add and one min per candidate."""
    assert bench.FLOOR_BYTES_PER_CELL == 4 + 1 and bench.FLOOR_OPS_PER_EVAL == 2
    assert bench.PEAK_VALU_OPS == 256 * 4 * 16 * 2.4e9
