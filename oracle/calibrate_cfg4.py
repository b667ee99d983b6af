"""Finds the slot-granularity factor g_b of each chain of benchmark configuration 4.

The recipe of that configuration asks for about 30 % infeasible (s, t, m) cells per
chain.  This script bisects g_b on the oracle's minimum-feasible-memory recursion and
prints the tuple frozen in workloads/chains.py (CFG4_G).  It calls only oracle/ and the
input generators.  Usage: python -m oracle.calibrate_cfg4
"""
import numpy as np

from oracle import oracle
from workloads.chains import CONFIGS, cfg4_raw_chains, scale_sizes


def main(target=0.30):
    c = CONFIGS[4]
    out = []
    for b, (uf, ub, x, xbar) in enumerate(cfg4_raw_chains(c["L"], c["B"], c["seed"])):
        lo, hi = 0.5, 3.0
        for _ in range(14):
            g = 0.5 * (lo + hi)
            xs, xbs = scale_sizes(x, xbar, g)
            frac = oracle.infeasible_fraction(c["L"], c["M"], xs, xbs)
            lo, hi = (g, hi) if frac < target else (lo, g)
        g = round(0.5 * (lo + hi), 4)
        xs, xbs = scale_sizes(x, xbar, g)
        frac = oracle.infeasible_fraction(c["L"], c["M"], xs, xbs)
        print(f"chain {b}: g = {g:.4f}  infeasible fraction = {frac:.4f}", flush=True)
        out.append(g)
    print("CFG4_G =", tuple(out))


if __name__ == "__main__":
    main()
