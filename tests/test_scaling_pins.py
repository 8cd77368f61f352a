"""Pins for the Eq. (2) / Amdahl oracle (Section 4.2, Section 1)."""
import os
from fractions import Fraction

import pytest

from oracle import partition as op
from oracle import scaling as osc
from paper_1712_02546_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "amdahl_bounds.txt")


def golden():
    out = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        key, val = line.split(":")
        out[key.strip()] = Fraction(val.strip())
    return out


def test_amdahl_figures_of_the_paper():
    g = golden()
    assert osc.amdahl_limit(g["conv_fraction_low"]) == g["limit_low"]
    assert osc.amdahl_limit(g["conv_fraction_high"]) == g["limit_high"]
    assert abs(osc.amdahl_limit(1 - g["other_fraction"]) - g["limit_about"]) <= g["limit_about_tolerance"]


def layer_of(cfg):
    assert cfg.H == cfg.W and cfg.R == cfg.S and cfg.P == cfg.Q
    return (cfg.H, cfg.C, cfg.R, cfg.K, cfg.P)


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3"])
def test_eq2_counts_the_three_tensors_of_a_layer(name):
    """in^2*inCh*batch, k^2*numK*inCh and out^2*numK*batch are the sizes of x, w and y."""
    cfg = synth.CONFIGS[name]
    x, w, dy = synth.make_inputs(cfg)
    assert osc.upload_elements([layer_of(cfg)], cfg.N) == x.size + w.size + dy.size


def test_eq2_is_additive_over_layers_and_linear_in_batch_for_the_map_terms():
    c1 = (32, 3, 5, 500, 28)      # the two convolutional layers of the largest network (Section 4.1)
    c2 = (14, 500, 5, 1500, 10)
    both = osc.upload_elements([c1, c2], 1024)
    assert both == osc.upload_elements([c1], 1024) + osc.upload_elements([c2], 1024)
    kernels = 25 * 500 * 3 + 25 * 1500 * 500
    assert osc.upload_elements([c1, c2], 0) == kernels
    assert both - kernels == 16 * (osc.upload_elements([c1, c2], 64) - kernels)
    # written out by hand for the second layer, batch 128
    assert osc.upload_elements([c2], 128) == 12_544_000 + 18_750_000 + 19_200_000


def test_partition_traffic_reduces_to_eq2_and_grows_with_devices():
    layer, batch = (14, 500, 5, 1500, 10), 128
    # one slave holding every kernel, the master none: exactly Eq. (2)
    assert osc.partition_elements(layer, batch, [0, 0, 1500], master=0) == osc.upload_elements([layer], batch)
    # n equal devices: (n-1) input broadcasts plus the slaves' share of kernels and maps
    for n in (2, 3, 4, 8):
        b = op.bounds([1] * n, 1500)
        got = osc.partition_elements(layer, batch, b, master=0)
        away = 1500 - (b[1] - b[0])
        assert got == (n - 1) * 196 * 500 * batch + away * (25 * 500 + 100 * batch)
    # a master that keeps everything sends only the inputs
    assert osc.partition_elements(layer, batch, [0, 1500, 1500], master=0) == 196 * 500 * batch


def test_transfer_time_of_the_papers_link():
    # doubles over about 5 Mbps (Section 4.2): one million elements take 12.8 s
    assert osc.transfer_seconds(1_000_000, 8, 5_000_000) == Fraction(64, 5)


def test_batch_time_and_speedup_model():
    # the worked example of Section 3.1.1 with free communication and no other layers: 1.5x
    w = op.shares([10, 20])
    assert osc.batch_seconds([10, 20], w, 0, 0) == Fraction(20, 3)
    assert osc.speedup([10, 20], w, 0, 0) == Fraction(3, 2)
    # with other layers the speed-up stays below Amdahl's limit and approaches it with many equal devices
    t_comp, t_conv = Fraction(13), Fraction(87)
    limit = osc.amdahl_limit(Fraction(87, 100))
    prev = 0
    for n in (1, 2, 4, 8, 64, 4096):
        s = osc.speedup([t_conv] * n, op.shares([1] * n), t_comp, 0)
        assert prev < s < limit
        prev = s
    assert limit - prev < Fraction(1, 10)
    # communication only ever costs
    assert osc.speedup([10, 20], w, 1, 2) < osc.speedup([10, 20], w, 1, 0)
