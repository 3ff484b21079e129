"""Mixing-matrix view of the gossip topologies (Section 3.2 of the paper, Theorems 1 and 2).

One round with peer table d mixes the workers with M = (I + P_d) / 2, where P_d[i, d[i]] = 1.
For the fair topology P_d is a permutation matrix, so M is doubly stochastic; without fair
selection M is only row-stochastic.  The paper studies the running product M_k ... M_1:
its second largest eigenvalue (bound on the averaging error) and the "imbalance factor",
the variance of the entries of the product minus the AllReduce matrix (all entries 1/n).

Host-only analysis on top of cx_topology_gen (NumPy linear algebra on n x n matrices);
nothing here touches the GPU.  `python -m paper_2012_15198_amd.mixing_analysis --n 16`
prints the two curves for the three topologies.
"""
from __future__ import annotations

import argparse
import json

import numpy as np

from . import cxmix

MODES = {"fair": 0, "directed_exponential": 1, "unfair": 2}


def mixing_matrix(peers_row: np.ndarray) -> np.ndarray:
    """(I + P)/2 with P[i, peers_row[i]] = 1: row i keeps half and receives half from its peer."""
    n = len(peers_row)
    m = 0.5 * np.eye(n)
    m[np.arange(n), np.asarray(peers_row)] += 0.5
    return m


def running_products(tables: np.ndarray):
    """Yields M_k ... M_1 for k = 1..K; tables is int [K][n] (one segment's table per round)."""
    prod = np.eye(tables.shape[1])
    for row in tables:
        prod = mixing_matrix(row) @ prod
        yield prod


def second_eigenvalue(m: np.ndarray) -> float:
    """Second largest eigenvalue modulus (the largest is 1 for a stochastic matrix)."""
    ev = np.sort(np.abs(np.linalg.eigvals(m)))[::-1]
    return float(ev[1]) if len(ev) > 1 else 0.0


def imbalance_factor(m: np.ndarray) -> float:
    """Variance of the entries of m - M_AR, M_AR being the all-1/n AllReduce matrix."""
    n = m.shape[0]
    return float(np.var(m - 1.0 / n))


def analyse(seed: int, n: int, rounds: int, mode: str = "fair", segment: int = 0) -> dict:
    """lambda_2 and imbalance factor of the running product over `rounds` rounds."""
    tables = cxmix.cx_topology_gen(seed, n, segment + 1, 0, rounds, MODES[mode])[:, segment, :]
    lam, imb = [], []
    for prod in running_products(tables):
        lam.append(second_eigenvalue(prod))
        imb.append(imbalance_factor(prod))
    return {"mode": mode, "n": n, "lambda2": lam, "imbalance": imb}


def main() -> None:
    ap = argparse.ArgumentParser(description=__doc__.splitlines()[0])
    ap.add_argument("--n", type=int, default=16)
    ap.add_argument("--rounds", type=int, default=24)
    ap.add_argument("--seed", type=int, default=1)
    ap.add_argument("--trials", type=int, default=20, help="seeds averaged per curve")
    args = ap.parse_args()
    out = {}
    for mode in MODES:
        runs = [analyse(args.seed + t, args.n, args.rounds, mode) for t in range(args.trials)]
        out[mode] = {"lambda2": np.mean([r["lambda2"] for r in runs], axis=0).round(6).tolist(),
                     "imbalance": np.mean([r["imbalance"] for r in runs], axis=0).round(9).tolist()}
    print(json.dumps({"n": args.n, "rounds": args.rounds, "trials": args.trials, **out}))


if __name__ == "__main__":
    main()
