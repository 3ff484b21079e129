#!/usr/bin/env python3
"""Writes tests/golden/topology_seed2_n8.txt: peer tables of the frozen topology spec
(Algorithm 2 of the paper: sequential fair draw, dead-end swap, counter-based draws keyed by seed,
round and segment), computed by the CPU oracle
ONLY.  The library's generator is tested against this file, so a change that alters both
sides in the same way is still caught.

    python tests/golden/make_topology_golden.py
"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle as O  # noqa: E402

CASES = [  # (seed, n, S, round0, R, mode)
    (2, 8, 4, 0, 3, 0), (2, 8, 2, 5, 2, 1), (2, 8, 2, 0, 2, 2), (2**64 - 1, 5, 3, 7, 2, 0), (2, 8, 3, 1, 1, 16)]


KEY_CASES = [  # (seed, round, segment): the pairs (1, 2) / (2, 1) and (0, 3) / (3, 0) tell round from segment
    (0, 0, 0), (2, 0, 0), (2, 1, 2), (2, 2, 1), (2, 0, 3), (2, 3, 0), (2**64 - 1, 7, 2), (42, 2**31 - 1, 4095)]


def key_vectors():
    """tests/golden/key_draw_vectors.txt: the 64-bit key of a (seed, round, segment) topology and its
    draws number 0, 1, 5 and 1024, as the oracle computes them."""
    with open(os.path.join(HERE, "key_draw_vectors.txt"), "w") as f:
        f.write("# Counter-based draws of the frozen topology spec, written by tests/golden/make_topology_golden.py\n")
        f.write("# from oracle/ alone.  seed round segment : key draw0 draw1 draw5 draw1024 (hexadecimal)\n")
        for seed, rnd, seg in KEY_CASES:
            k = O.key(seed, rnd, seg)
            f.write(f"{seed} {rnd} {seg} : {k:016x} " + " ".join(f"{O.draw(k, i):016x}" for i in (0, 1, 5, 1024)) + "\n")


def main():
    key_vectors()
    with open(os.path.join(HERE, "topology_seed2_n8.txt"), "w") as f:
        f.write("# Peer tables written by tests/golden/make_topology_golden.py from oracle/ alone.\n")
        f.write("# One line per (case, round, segment): seed n S round segment mode : receive-from row of 0..n-1\n")
        for seed, n, S, r0, R, mode in CASES:
            t = O.topology(seed, n, S, r0, R, mode)
            for r in range(R):
                for s in range(S):
                    f.write(f"{seed} {n} {S} {r0 + r} {s} {mode} : {' '.join(map(str, t[r, s]))}\n")


if __name__ == "__main__":
    main()
