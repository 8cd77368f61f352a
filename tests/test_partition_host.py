"""conv_partition / conv_partition_estimate (host code of the C-ABI library) against the
exact-rational oracle of Eq. (1), Section 3.1.1.  No GPU is touched."""
import os
import random
from fractions import Fraction

import pytest

import paper_1712_02546_amd as cs
from oracle import partition as op

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "eq1_worked_example.txt")


def test_worked_example_through_the_abi():
    shares, bounds = cs.conv_partition([10.0, 20.0], 1500)
    assert shares == pytest.approx([2 / 3, 1 / 3], rel=1e-15)
    assert bounds == [0, 1000, 1500]
    finish, speedup = cs.conv_partition_estimate([10.0, 20.0], shares)
    assert f"{finish:.2f}" == "6.67"
    assert speedup == pytest.approx(1.5, rel=1e-14)
    # the equal split of the example: 5 s and 10 s, slower than device 1 alone is fast
    finish, speedup = cs.conv_partition_estimate([10.0, 20.0], [0.5, 0.5])
    assert finish == 10.0 and speedup == 1.0


@pytest.mark.parametrize("seed", range(40))
def test_random_times_match_the_oracle(seed):
    rng = random.Random(seed)
    n = rng.randint(1, 12)
    t = [rng.uniform(0.05, 40.0) for _ in range(n)]
    K = rng.choice([0, 1, 7, 96, 500, 1500, 4096, 100000])
    shares, bounds = cs.conv_partition(t, K)
    want = op.shares(t)
    assert all(abs(Fraction(a) - b) <= Fraction(1, 10 ** 14) for a, b in zip(shares, want))
    assert bounds == op.bounds(t, K)           # integer work: exact
    fin, sp = cs.conv_partition_estimate(t, shares)
    assert fin == pytest.approx(float(max(op.finish_times(t, want))), rel=1e-13)
    assert sp == pytest.approx(float(op.speedup(t, want)), rel=1e-13)


@pytest.mark.parametrize("t,K", [
    ([1, 1, 1], 4), ([1, 1, 1], 5), ([2, 2], 1), ([3.5] * 7, 100), ([10, 20], 100), ([10, 20], 101),
    ([1, 2, 4], 7), ([1, 2, 4], 1000), ([5, 5, 10, 10], 9), ([0.1] * 64, 63), ([1, 3], 0),
])
def test_ties_and_exact_quotas_match_the_oracle(t, K):
    assert cs.conv_partition(t, K)[1] == op.bounds(t, K)


def test_paper_cluster_sizes():
    # three and four devices as in the experiments (Section 4): shares sum to one, bounds cover K
    for t in ([1.0, 1.3, 2.1], [0.8, 1.0, 1.7, 2.4]):
        for K in (50, 500, 1500):
            shares, bounds = cs.conv_partition(t, K)
            assert sum(shares) == pytest.approx(1.0, abs=1e-15)
            assert bounds[0] == 0 and bounds[-1] == K and bounds == sorted(bounds)
            assert bounds == op.bounds(t, K)


@pytest.mark.parametrize("t,K,code", [
    ([], 10, -1), ([1.0, 0.0], 10, -9), ([1.0, -1.0], 10, -9), ([float("nan")], 10, -9),
    ([float("inf"), 1.0], 10, -9), ([1.0], -1, -9), ([1.0] * 65, 10, -9),
])
def test_bad_partition_arguments(t, K, code):
    assert cs.conv_partition(t, K, raw_status=True) == code


def test_estimate_rejects_bad_shares():
    assert cs.conv_partition_estimate([1.0, 2.0], [0.5, -0.5], raw_status=True) == -9
    assert cs.conv_partition_estimate([1.0, 0.0], [0.5, 0.5], raw_status=True) == -9


class FakeBuf:
    """Stands in for a device tensor: the calls below must fail before using it."""

    def __init__(self, ptr, nbytes=1 << 20):
        self._p, self._n = ptr, nbytes

    def data_ptr(self):
        return self._p

    def numel(self):
        return self._n

    def element_size(self):
        return 1


LAYER = dict(N=8, C=3, H=32, W=32, K=16, R=5, S=5)
A = FakeBuf(0x10000)
WS = FakeBuf(0x20000, 1 << 30)


@pytest.mark.parametrize("fn", [cs.conv_layer_fwd, cs.conv_layer_bwd_data, cs.conv_layer_bwd_weight])
@pytest.mark.parametrize("bounds,code", [
    ([1, 16], -9), ([0, 15], -9), ([0, 9, 8, 16], -9), ([0, 17], -9), ([0] + [16] * 65, -9),
])
def test_layer_calls_reject_bad_bounds(fn, bounds, code):
    assert fn(cs.ConvDesc(**LAYER), bounds, A, A, A, WS, stream=0, raw_status=True) == code


@pytest.mark.parametrize("fn", [cs.conv_layer_fwd, cs.conv_layer_bwd_data, cs.conv_layer_bwd_weight])
def test_layer_calls_reject_bad_layers_null_pointers_and_small_workspaces(fn):
    good = [0, 4, 4, 16]
    assert fn(cs.ConvDesc(**{**LAYER, "N": 0}), good, A, A, A, WS, stream=0, raw_status=True) == -2
    assert fn(cs.ConvDesc(**LAYER), good, None, A, A, WS, stream=0, raw_status=True) == -1
    assert fn(cs.ConvDesc(**LAYER), good, A, A, None, WS, stream=0, raw_status=True) == -1
    assert fn(cs.ConvDesc(**LAYER), good, A, A, A, FakeBuf(0x20000, 256), stream=0, raw_status=True) == -5


def test_layer_workspace_is_the_sum_or_the_maximum_of_the_slices():
    d = cs.ConvDesc(**LAYER)
    bounds = [0, 4, 4, 16]

    def r256(b):
        return (b + 255) // 256 * 256

    per = {p: [r256(cs.conv_workspace_bytes(cs.ConvDesc(**LAYER, k0=a, k1=b), p))
               for a, b in zip(bounds, bounds[1:]) if b > a]
           for p in (cs.PASS_FWD, cs.PASS_BWD_DATA, cs.PASS_BWD_WEIGHT)}
    assert cs.conv_layer_workspace_bytes(d, bounds, cs.PASS_FWD) == sum(per[cs.PASS_FWD])
    assert cs.conv_layer_workspace_bytes(d, bounds, cs.PASS_BWD_WEIGHT) == sum(per[cs.PASS_BWD_WEIGHT])
    assert cs.conv_layer_workspace_bytes(d, bounds, cs.PASS_BWD_DATA) == max(per[cs.PASS_BWD_DATA])
    assert cs.conv_layer_workspace_bytes(d, [0, 3], cs.PASS_FWD) == 0      # bounds do not end at K


def test_calibrate_argument_checks():
    d = cs.ConvDesc(**LAYER)
    assert cs.conv_calibrate_workspace_bytes(d, 0) > 0
    assert cs.conv_calibrate_workspace_bytes(d, 7) > cs.conv_calibrate_workspace_bytes(d, 1)
    assert cs.conv_calibrate_workspace_bytes(d, 8) == 0
    assert cs.conv_calibrate(d, 8, 1, WS, stream=0, raw_status=True) == -8
    assert cs.conv_calibrate(d, 1, 0, WS, stream=0, raw_status=True) == -2
    assert cs.conv_calibrate(cs.ConvDesc(**LAYER, k0=3, k1=3), 1, 1, WS, stream=0, raw_status=True) == -3
    assert cs.conv_calibrate(d, 1, 1, FakeBuf(0x20000, 1024), stream=0, raw_status=True) == -5
