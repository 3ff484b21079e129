#!/usr/bin/env python3
"""Writes tests/golden/mixing_curves_n16.json: the two curves of the paper's mixing-matrix study
(Section 3.2: second largest eigenvalue of the running product M_k ... M_1 and its "imbalance factor",
the variance of the entries of the product minus the all-1/n AllReduce matrix) for n = 16 workers,
24 rounds, averaged over 20 seeds, for the fair random topology (Algorithm 2), the random topology
without fair peer selection and the directed exponential graph.  The paper's own figure values are lost
with its figures; this file freezes what the frozen topology spec produces.  Topologies come from
oracle/ ONLY; the linear algebra is NumPy's, written out here.

    python tests/golden/make_mixing_curves.py
"""
import json
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle as O  # noqa: E402

N, ROUNDS, TRIALS, SEED = 16, 24, 20, 1
MODES = {"fair": 0, "directed_exponential": 1, "unfair": 2}


def curves(seed, mode):
    tables = O.topology(seed, N, 1, 0, ROUNDS, mode)[:, 0, :]
    prod = np.eye(N)
    lam, imb = [], []
    for d in tables:
        m = 0.5 * np.eye(N)
        m[np.arange(N), d] += 0.5               # row i keeps half and receives half from d[i]
        prod = m @ prod
        lam.append(float(np.sort(np.abs(np.linalg.eigvals(prod)))[::-1][1]))
        imb.append(float(np.var(prod - 1.0 / N)))
    return lam, imb


def main():
    out = {"n": N, "rounds": ROUNDS, "trials": TRIALS, "seed": SEED}
    for name, mode in MODES.items():
        runs = [curves(SEED + t, mode) for t in range(TRIALS)]
        out[name] = {"lambda2": np.mean([r[0] for r in runs], axis=0).round(9).tolist(),
                     "imbalance": np.mean([r[1] for r in runs], axis=0).round(12).tolist()}
    with open(os.path.join(HERE, "mixing_curves_n16.json"), "w") as f:
        json.dump(out, f, indent=1)
        f.write("\n")


if __name__ == "__main__":
    main()
