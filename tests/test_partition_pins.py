"""Pins for the Eq. (1) partition oracle: the paper's worked example, closed forms,
invariants and brute force (Section 3.1.1)."""
import itertools
import os
import random
from fractions import Fraction

import pytest

from oracle import partition as op

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "eq1_worked_example.txt")


def golden():
    out = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        key, val = line.split(":")
        out[key.strip()] = val.split()
    return out


def test_worked_example_of_the_paper():
    g = golden()
    t = [int(v) for v in g["times_s"]]
    assert op.performance(t) == [Fraction(v) for v in g["performance"]]
    w = op.shares(t)
    assert w == [Fraction(v) for v in g["shares"]]
    fin = op.finish_times(t, w)
    assert fin[0] == fin[1]
    assert f"{float(fin[0]):.2f}" == g["finish_s_rounded_2"][0]
    assert op.speedup(t, w) == Fraction(g["speedup"][0])
    # the equal split the example starts from: 5 s and 10 s, no gain over device 1 alone
    eq = op.finish_times(t, [Fraction(1, 2)] * 2)
    assert eq == [Fraction(v) for v in g["equal_split_finish_s"]]
    assert op.speedup(t, [Fraction(1, 2)] * 2) <= Fraction(g["equal_split_speedup_not_above"][0])


def test_shares_closed_form_harmonic():
    # max(t) cancels: w_i = (1/t_i) / sum_j (1/t_j)
    t = [3, 7, 11, 2]
    inv = [Fraction(1, v) for v in t]
    assert op.shares(t) == [v / sum(inv) for v in inv]


@pytest.mark.parametrize("seed", range(20))
def test_share_invariants(seed):
    rng = random.Random(seed)
    n = rng.randint(1, 9)
    t = [Fraction(rng.randint(1, 1000), rng.randint(1, 50)) for _ in range(n)]
    w = op.shares(t)
    assert sum(w) == 1 and all(v > 0 for v in w)
    fin = op.finish_times(t, w)
    assert len(set(fin)) == 1                      # everybody finishes together
    scale = Fraction(rng.randint(1, 99), 7)
    assert op.shares([v * scale for v in t]) == w  # units of time do not matter
    for i, j in itertools.combinations(range(n), 2):
        assert w[i] * t[i] == w[j] * t[j]          # share inversely proportional to time
    perm = list(range(n))
    rng.shuffle(perm)
    wp = op.shares([t[i] for i in perm])
    assert wp == [w[i] for i in perm]


def test_equal_devices_get_equal_shares_and_slower_gets_less():
    assert op.shares([4.0] * 5) == [Fraction(1, 5)] * 5
    w = op.shares([1, 2, 4])
    assert w[0] > w[1] > w[2] and w == [Fraction(4, 7), Fraction(2, 7), Fraction(1, 7)]


def test_single_device_owns_everything():
    assert op.shares([123.0]) == [1]
    assert op.bounds([0.5], 77) == [0, 77]


def test_kernel_counts_of_the_worked_example():
    # K divisible by 3: exact thirds; otherwise the larger remainder wins
    assert op.kernel_counts([10, 20], 1500) == [1000, 500]
    assert op.kernel_counts([10, 20], 100) == [67, 33]      # quotas 66.67 / 33.33
    assert op.kernel_counts([10, 20], 101) == [67, 34]      # quotas 67.33 / 33.67
    assert op.bounds([10, 20], 1500) == [0, 1000, 1500]


def _brute_force_counts(t, K):
    """All integer vectors summing to K; keep those that deviate least from the quotas in
    the max norm, then least in the sum of squares, then the lexicographically largest
    (which is what 'ties go to the lower index' produces)."""
    n = len(t)
    quota = [w * K for w in op.shares(t)]
    best = None
    for c in itertools.product(range(K + 1), repeat=n):
        if sum(c) != K:
            continue
        dev = [abs(a - q) for a, q in zip(c, quota)]
        key = (max(dev), sum(d * d for d in dev), tuple(-v for v in c))
        if best is None or key < best[0]:
            best = (key, c)
    return list(best[1])


@pytest.mark.parametrize("seed", range(12))
def test_kernel_counts_brute_force(seed):
    rng = random.Random(100 + seed)
    n = rng.randint(2, 4)
    t = [rng.randint(1, 9) for _ in range(n)]
    K = rng.randint(0, 9)
    assert op.kernel_counts(t, K) == _brute_force_counts(t, K)


@pytest.mark.parametrize("seed", range(20))
def test_kernel_count_invariants(seed):
    rng = random.Random(200 + seed)
    n = rng.randint(1, 8)
    t = [rng.uniform(0.1, 30.0) for _ in range(n)]
    K = rng.randint(0, 3000)
    c = op.kernel_counts(t, K)
    assert sum(c) == K and min(c) >= 0
    quota = [w * K for w in op.shares(t)]
    assert all(abs(a - q) < 1 for a, q in zip(c, quota))     # quota rule
    b = op.bounds(t, K)
    assert b[0] == 0 and b[-1] == K and all(b[i + 1] - b[i] == c[i] for i in range(n))
    # a faster device never gets fewer kernels than a slower one
    for i, j in itertools.combinations(range(n), 2):
        if t[i] < t[j]:
            assert c[i] >= c[j]


def test_ties_go_to_the_lower_index():
    assert op.kernel_counts([1, 1, 1], 4) == [2, 1, 1]
    assert op.kernel_counts([1, 1, 1], 5) == [2, 2, 1]
    assert op.kernel_counts([2, 2], 1) == [1, 0]


def test_rejects_bad_times():
    for bad in ([], [1, 0], [1, -2]):
        with pytest.raises(ValueError):
            op.shares(bad)
