"""Worker side of the full-size neighbour-table checks: the brute-force oracle for one block of
rows (imports nothing but the oracle, so that spawned worker processes start quickly and never
touch the GPU)."""
import numpy as np

from oracle import build_neighbours


def oracle_rows(args):
    E, k, lo, hi = args
    return lo, build_neighbours(E, k, rows=np.arange(lo, hi))
