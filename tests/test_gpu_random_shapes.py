"""Seeded sweep over small random layers (extents around the tile, chunk and image-block
boundaries, strides, paddings, rectangular filters, interior slices, both dtypes): the three
passes against the oracle, element by element."""
import random

import pytest

import oracle
import paper_1712_02546_amd as cs
from helpers import BF16_TOL, FP32_TOL, Device, oracle_shape, rel_err
from paper_1712_02546_amd import synth

pytestmark = pytest.mark.gpu


def random_case(seed):
    rng = random.Random(seed)
    while True:
        R = rng.choice([1, 1, 2, 3, 3, 5, 7])
        S = rng.choice([1, 2, 3, 3, 5, 4])
        stride = rng.choice([1, 1, 1, 2, 3])
        pad = rng.choice([0, 0, 1, 2, 3])
        H = rng.randint(max(R - 2 * pad, 1), 20)
        W = rng.randint(max(S - 2 * pad, 1), 20)
        N = rng.choice([1, 3, 8, 31, 32, 33, 64, 65, 96, 100, 128, 130, 160])
        C = rng.choice([1, 2, 3, 8, 31, 32, 33, 40, 64, 100, 129, 140])
        K = rng.choice([1, 2, 5, 16, 31, 32, 33, 64, 100, 127, 128, 129, 200, 300])
        if N * C * H * W * K * R * S > 2e9 or N * C * H * W > 3e6:
            continue
        k0 = rng.randint(0, K - 1)
        k1 = rng.randint(k0 + 1, K)
        if rng.random() < 0.4:
            k0, k1 = 0, K
        dtype = cs.CONV_BF16 if rng.random() < 0.3 else cs.CONV_F32
        cfg = synth.random_layer(2000 + seed, N=N, C=C, H=H, W=W, K=K, R=R, S=S, stride=stride, pad=pad, k0=k0, k1=k1)
        return cfg, dtype


@pytest.mark.parametrize("block", range(10))
def test_random_layers_match_oracle(block):
    for seed in range(block * 12, block * 12 + 12):
        cfg, dtype = random_case(seed)
        k0, k1 = cfg.slice
        x, w, dy = synth.make_inputs(cfg)
        if dtype == cs.CONV_BF16:
            x, w, dy = (synth.round_to_bf16(a) for a in (x, w, dy))
        sh = oracle_shape(cfg)
        dev = Device(cfg, x, w, dy, dtype=dtype)
        tol = FP32_TOL if dtype == cs.CONV_F32 else BF16_TOL
        what = f"seed {seed}: {cfg} dtype {dtype}"
        assert rel_err(dev.fwd(fill=0.0)[:, k0:k1], oracle.conv_fwd(sh, x, w)[:, k0:k1]) <= tol, "y, " + what
        assert rel_err(dev.bwd_data(), oracle.conv_bwd_data(sh, dy, w)) <= tol, "dx, " + what
        assert rel_err(dev.bwd_weight(fill=0.0)[k0:k1], oracle.conv_bwd_weight(sh, x, dy)[k0:k1]) <= FP32_TOL, \
            "dw, " + what
