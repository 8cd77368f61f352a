"""conv_comm_elements / conv_comm_elements_partition / conv_scaling_estimate (host code of the
C-ABI library) against the exact oracle of Eq. (2) and Section 4.2.  No GPU is touched."""
import math
import random
from fractions import Fraction

import pytest

import paper_1712_02546_amd as cs
from oracle import partition as op
from oracle import scaling as osc

C1 = (32, 3, 5, 500, 28)
C2 = (14, 500, 5, 1500, 10)


def test_eq2_matches_the_oracle_exactly():
    rng = random.Random(7)
    for _ in range(30):
        layers = [(rng.randint(1, 300), rng.randint(1, 600), rng.randint(1, 11), rng.randint(1, 2000),
                   rng.randint(1, 300)) for _ in range(rng.randint(0, 4))]
        batch = rng.choice([0, 1, 64, 128, 1024, 50000])
        assert cs.conv_comm_elements(layers, batch) == osc.upload_elements(layers, batch)   # integers < 2^53
    assert cs.conv_comm_elements([C1, C2], 1024) == osc.upload_elements([C1, C2], 1024)


def test_partition_traffic_matches_the_oracle_exactly():
    rng = random.Random(8)
    for _ in range(30):
        n = rng.randint(1, 9)
        t = [rng.uniform(0.5, 9.0) for _ in range(n)]
        layer = rng.choice([C1, C2])
        batch = rng.choice([64, 128, 1024])
        bounds = op.bounds(t, layer[3])
        master = rng.randrange(n)
        want = osc.partition_elements(layer, batch, bounds, master)
        assert cs.conv_comm_elements_partition(layer, batch, bounds, master) == want
    assert cs.conv_comm_elements_partition(C2, 128, [0, 0, 1500], 0) == cs.conv_comm_elements([C2], 128)


def test_estimate_matches_the_oracle():
    rng = random.Random(9)
    for _ in range(30):
        n = rng.randint(1, 8)
        t = [rng.uniform(0.5, 9.0) for _ in range(n)]
        w = op.shares(t)
        t_comp = rng.uniform(0.0, 3.0)
        elements = osc.partition_elements(C2, 128, op.bounds(t, 1500), 0)
        sec, sp, am = cs.conv_scaling_estimate(t, [float(v) for v in w], t_comp, elements, 8, 5e6)
        comm = osc.transfer_seconds(elements, 8, 5_000_000)
        want = osc.batch_seconds(t, w, Fraction(t_comp), comm)
        assert sec == pytest.approx(float(want), rel=1e-13)
        assert sp == pytest.approx(float(osc.speedup(t, w, Fraction(t_comp), comm)), rel=1e-13)
        frac = Fraction(t[0]) / (Fraction(t[0]) + Fraction(t_comp))
        assert am == pytest.approx(float(osc.amdahl_limit(frac)), rel=1e-12)


def test_figures_of_the_paper_through_the_abi():
    # worked example of Section 3.1.1: free communication, no other layers -> 6.67 s, 1.5x, no Amdahl bound
    sec, sp, am = cs.conv_scaling_estimate([10, 20], [2 / 3, 1 / 3], 0.0, 0.0, 8, 5e6)
    assert f"{sec:.2f}" == "6.67" and sp == pytest.approx(1.5) and math.isinf(am)
    # Section 1: 60 % .. 90 % convolution -> bounds 2.5 .. 10; Section 4.2: 13 % other layers -> about 7.7
    assert cs.conv_scaling_estimate([60], [1.0], 40, 0, 8, 5e6)[2] == pytest.approx(2.5)
    assert cs.conv_scaling_estimate([90], [1.0], 10, 0, 8, 5e6)[2] == pytest.approx(10.0)
    assert abs(cs.conv_scaling_estimate([87], [1.0], 13, 0, 8, 5e6)[2] - 7.76) < 0.1
    # one million doubles over 5 Mbps take 12.8 s
    assert cs.conv_scaling_estimate([1], [1.0], 0, 1e6, 8, 5e6)[0] == pytest.approx(1 + 12.8)


def test_bad_arguments():
    assert cs.conv_comm_elements([(-1, 3, 5, 16, 28)], 8, raw_status=True) == -2
    assert cs.conv_comm_elements([C1], -1, raw_status=True) == -2
    assert cs.conv_comm_elements_partition(C2, 128, [0, 700, 1400], 0, raw_status=True) == -9
    assert cs.conv_comm_elements_partition(C2, 128, [0, 700, 1500], 2, raw_status=True) == -9
    assert cs.conv_scaling_estimate([1, 2], [0.5, 0.5], 0, 0, 8, 0.0, raw_status=True) == -9
    assert cs.conv_scaling_estimate([1, 0], [0.5, 0.5], 0, 0, 8, 1e6, raw_status=True) == -9
    assert cs.conv_scaling_estimate([1, 2], [0.5, 0.5], 0, 0, 8, 1e6, master=2, raw_status=True) == -9
