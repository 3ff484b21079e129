"""Pins for the oracle's topology generator (Algorithm 2 of the paper and the
readings of its silent points).  CPU only."""
import itertools
import math
import os
from collections import Counter
from fractions import Fraction

import numpy as np
import pytest

import oracle as O

GAMMA = 0x9E3779B97F4A7C15
M64 = 2**64 - 1


def test_mixer_matches_published_splitmix64_vectors(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "splitmix64_vectors.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) >= 4
    for k, val in rows:
        assert O.mix64((int(k) * GAMMA) & M64) == int(val, 16)


def test_key_and_draw_are_counter_based():
    # distinct (round, segment, index) give distinct draws; same inputs repeat
    seen = set()
    for r in range(6):
        for s in range(6):
            k = O.key(42, r, s)
            assert k == O.key(42, r, s)
            for i in range(6):
                seen.add(O.draw(k, i))
    assert len(seen) == 6 * 6 * 6
    assert O.key(42, 1, 2) != O.key(43, 1, 2) != O.key(42, 2, 1)


def _mix(z):
    """The bit mixer in Python integers: xor-shift 30, multiply, xor-shift 27, multiply, xor-shift 31."""
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
    return z ^ (z >> 31)


def _key(seed, rnd, seg):
    """The frozen key function, from its statement: mix(mix(mix(seed + gamma) + round) + segment)."""
    return _mix((_mix((_mix((seed + GAMMA) & M64) + rnd) & M64) + seg) & M64)


def test_key_and_draw_printed_vectors(golden_dir):
    """The key of a (seed, round, segment) topology and its draws, recomputed here in Python integers
    from the statement of the generator and compared with the stored vectors and with the oracle.  The
    vectors hold (round, segment) = (1, 2) next to (2, 1): swapping the two fields fails."""
    rows = [l for l in open(os.path.join(golden_dir, "key_draw_vectors.txt")) if not l.startswith("#")]
    assert len(rows) >= 8
    keys = {}
    for line in rows:
        head, tail = line.split(":")
        seed, rnd, seg = map(int, head.split())
        k, *draws = (int(h, 16) for h in tail.split())
        assert _key(seed, rnd, seg) == k == O.key(seed, rnd, seg), line
        for i, want in zip((0, 1, 5, 1024), draws):
            assert _mix((k + i) & M64) == want == O.draw(k, i), (line, i)
        keys[(seed, rnd, seg)] = k
    assert keys[(2, 1, 2)] != keys[(2, 2, 1)] and keys[(2, 0, 3)] != keys[(2, 3, 0)]
    assert len(set(keys.values())) == len(keys)


def test_tables_follow_from_the_python_integer_draws():
    """Algorithm 2 walked in Python from draws computed in Python integers (no oracle call inside)
    gives the oracle's tables, for several rounds and segments: the oracle's indexing of round and
    segment into the key, and of the rank into the draw, is the stated one."""
    def table(seed, rnd, seg, n):
        k = _key(seed, rnd, seg)
        chosen, d = [], []
        for i in range(n):
            cand = [j for j in range(n) if j != i and j not in chosen]
            if not cand:
                swap = (_mix((k + n) & M64) * (n - 1)) >> 64
                d.append(d[swap])
                d[swap] = i
                break
            pick = cand[(_mix((k + i) & M64) * len(cand)) >> 64]
            chosen.append(pick)
            d.append(pick)
        return d
    for seed, n, S, r0, R in [(2, 8, 4, 0, 3), (5, 3, 6, 4, 30), (2**64 - 1, 13, 2, 9, 2)]:
        got = O.topology(seed, n, S, r0, R)
        for r in range(R):
            for s in range(S):
                assert got[r, s].tolist() == table(seed, r0 + r, s, n), (seed, r, s)


def test_uniform_is_floor_of_scaled_product():
    for v, m in [(0, 7), (M64, 7), (2**63, 2), (2**63 - 1, 2), (12345678901234567890, 255),
                 (2**64 // 3, 3), (2**64 // 3 + 1, 3)]:
        assert O.uniform(v, m) == (v * m) >> 64
        assert 0 <= O.uniform(v, m) < m


def _trace(key, n):
    """Algorithm 2 walked by hand from the raw draws (candidate lists in ascending
    rank order; the last rank swaps with an earlier one if only itself is left)."""
    chosen, d = [], []
    for i in range(n):
        cand = [j for j in range(n) if j != i and j not in chosen]
        if not cand:
            k = (O.draw(key, n) * (n - 1)) >> 64
            d.append(d[k])
            d[k] = i
            break
        pick = cand[(O.draw(key, i) * len(cand)) >> 64]
        chosen.append(pick)
        d.append(pick)
    return d


@pytest.mark.parametrize("n", [2, 3, 4, 5, 6, 7, 8, 16, 33, 64, 256])
def test_fair_draw_follows_hand_trace_and_is_a_derangement(n):
    for r in range(40):
        key = O.key(1234 + n, r, r % 5)
        d = O.fair_draw(key, n).tolist()
        assert d == _trace(key, n)
        assert sorted(d) == list(range(n)), "every rank is received from exactly once"
        assert all(d[i] != i for i in range(n)), "zero diagonal: nobody pairs with itself"


def test_n2_is_always_the_swap():
    for r in range(50):
        assert O.fair_draw(O.key(9, r, 0), 2).tolist() == [1, 0]


def _exact_distribution(n):
    """Exact probability of every table under Algorithm 2 + the swap rule,
    by walking the whole draw tree in rational arithmetic."""
    dist = Counter()

    def rec(i, d, p):
        if i == n:
            dist[tuple(d)] += p
            return
        cand = [j for j in range(n) if j != i and j not in d]
        if not cand:
            for k in range(n - 1):
                e = list(d)
                e.append(e[k])
                e[k] = i
                dist[tuple(e)] += p / (n - 1)
            return
        for j in cand:
            rec(i + 1, d + [j], p / len(cand))

    rec(0, [], Fraction(1))
    return dist


def test_exact_tree_n3_is_three_eighths_five_eighths():
    dist = _exact_distribution(3)
    assert dist == {(1, 2, 0): Fraction(3, 8), (2, 0, 1): Fraction(5, 8)}


@pytest.mark.parametrize("n,samples", [(3, 40000), (4, 40000), (5, 60000), (6, 120000)])
def test_generator_matches_exact_tree_chi_square(n, samples):
    dist = _exact_distribution(n)
    assert sum(dist.values()) == 1
    # every derangement and nothing else is reachable
    derangements = [p for p in itertools.permutations(range(n))
                    if all(p[i] != i for i in range(n))]
    assert set(dist) == set(derangements)
    S = 8
    R = samples // S
    tabs = O.topology(2024 + n, n, S, 0, R).reshape(-1, n)
    got = Counter(map(tuple, tabs.tolist()))
    assert set(got) <= set(dist)
    chi2 = sum((got.get(t, 0) - float(p) * len(tabs)) ** 2 / (float(p) * len(tabs))
               for t, p in dist.items())
    dof = len(dist) - 1
    # Wilson-Hilferty upper bound at ~4.5 sigma: fails for a wrong draw rule, never by chance
    bound = dof * (1 - 2 / (9 * dof) + 4.5 * math.sqrt(2 / (9 * dof))) ** 3 if dof > 0 else 1
    assert chi2 < max(bound, 25.0), (chi2, dof)


def test_dead_end_frequency_matches_tree():
    # P(dead end) at n=3 is 1/4 (first pick 1, second pick 0); the swap then makes
    # [2,0,1] (k=0) or [1,2,0] (k=1).  Check through the raw draws.
    n, hits, total = 3, 0, 20000
    for r in range(total):
        key = O.key(77, r, 3)
        first = [1, 2][(O.draw(key, 0) * 2) >> 64]
        if first == 1 and [0, 2][(O.draw(key, 1) * 2) >> 64] == 0:
            hits += 1
    assert abs(hits / total - 0.25) < 0.015


def test_tables_differ_between_segments_and_rounds():
    t = O.topology(5, 32, 8, 0, 50)
    flat = t.reshape(-1, 32)
    assert len({tuple(r) for r in flat.tolist()}) == len(flat)
    # a model-wise table (same for all segments) would contradict Section 3
    assert not all((t[0, s] == t[0, 0]).all() for s in range(8))


def test_resume_is_a_pure_function_of_round():
    a = O.topology(11, 16, 4, 0, 10)
    b = O.topology(11, 16, 4, 6, 4)
    assert (a[6:] == b).all()


def test_mixing_matrix_is_doubly_stochastic_and_products_flatten():
    # M = (I + Perm)/2 per segment; rows and columns sum to one (Section 3.2), and
    # the running product tends to the all-1/n matrix (Theorem 1).
    n = 16
    t = O.topology(3, n, 1, 0, 200)[:, 0]
    prod = np.eye(n)
    for d in t:
        M = 0.5 * np.eye(n)
        M[np.arange(n), d] += 0.5
        assert np.allclose(M.sum(0), 1) and np.allclose(M.sum(1), 1)
        prod = M @ prod
    assert np.abs(prod - 1.0 / n).max() < 1e-9


def test_directed_exponential_mode_by_hand():
    t = O.topology(0, 8, 2, 0, 4, mode=1)
    for r, hop in enumerate([1, 2, 4, 1]):
        for s in range(2):
            assert t[r, s].tolist() == [(i - hop) % 8 for i in range(8)]
    # n not a power of two: ceil(log2 6) = 3 distinct hops 1, 2, 4
    t6 = O.topology(0, 6, 1, 0, 3, mode=1)[:, 0]
    assert t6[2].tolist() == [2, 3, 4, 5, 0, 1]
    # n = 2: the only hop is 1
    assert O.topology(0, 2, 1, 5, 1, mode=1)[0, 0].tolist() == [1, 0]
