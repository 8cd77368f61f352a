"""Partitioned layer on the GPU (Section 3.1.1 and Algorithm 1): slices sized by Eq. (1) run
through conv_layer_* and must give the full layer's y, dx and dw of the oracle; the
calibration probe returns a plausible time."""
import numpy as np
import pytest

import oracle
import paper_1712_02546_amd as cs
from helpers import BF16_TOL, FP32_TOL, Device, desc_of, oracle_shape, rel_err
from oracle import partition as op
from paper_1712_02546_amd import synth

pytestmark = pytest.mark.gpu

SAME_MATH_TOL = 2e-5   # same sums in another order (fp32)


def check(got, ref, tol, what):
    e = rel_err(got, ref)
    assert e <= tol, f"{what}: max rel err {e:.3e} > {tol:.1e}"


def layer_ws(cfg, bounds, dtype):
    import torch
    need = max(cs.conv_layer_workspace_bytes(desc_of(cfg, dtype), bounds, p) for p in (0, 1, 2))
    return torch.empty(max(need, 256), dtype=torch.uint8, device="cuda:0")


def run_layer(dev, cfg, bounds, dtype, dx_init=None, accumulate=0):
    import torch
    ws = layer_ws(cfg, bounds, dtype)
    y = dev._empty((cfg.N, cfg.K, cfg.P, cfg.Q), fill=0.0)
    dw = dev._empty((cfg.K, cfg.C, cfg.R, cfg.S), fp32=True, fill=0.0)
    dx = dev._empty((cfg.N, cfg.C, cfg.H, cfg.W)) if dx_init is None else dev._up(dx_init)
    d = desc_of(cfg, dtype, accumulate)
    cs.conv_layer_fwd(d, bounds, dev.x, dev.w, y, ws)
    cs.conv_layer_bwd_data(d, bounds, dev.dy, dev.w, dx, ws)
    cs.conv_layer_bwd_weight(d, bounds, dev.x, dev.dy, dw, ws)
    torch.cuda.synchronize()
    return y.float().cpu().numpy(), dx.float().cpu().numpy(), dw.float().cpu().numpy()


CASES = [
    # (layer, probe times of the devices)
    (synth.random_layer(30, N=36, C=24, H=12, W=12, K=200, R=5, S=5, pad=1), [10.0, 20.0]),
    (synth.random_layer(31, N=40, C=48, H=11, W=13, K=150, R=3, S=3, stride=2, pad=1), [1.0, 1.3, 2.1]),
    (synth.random_layer(32, N=33, C=40, H=10, W=10, K=37, R=3, S=3), [0.8, 1.0, 1.7, 2.4]),
    (synth.random_layer(33, N=8, C=3, H=32, W=32, K=5, R=5, S=5), [1.0] * 8),      # more devices than kernels
    (synth.CONFIGS["cfg1"], [3.0, 1.0, 2.0, 1.0, 5.0, 1.0]),                        # six slices on four streams
]


@pytest.mark.parametrize("cfg,times", CASES, ids=lambda v: getattr(v, "name", None))
def test_partitioned_layer_matches_oracle_fp32(cfg, times):
    cfg = cfg.with_slice(0, cfg.K)
    x, w, dy = synth.make_inputs(cfg)
    _, bounds = cs.conv_partition(times, cfg.K)
    assert bounds == op.bounds(times, cfg.K)
    dev = Device(cfg, x, w, dy)
    y, dx, dw = run_layer(dev, cfg, bounds, cs.CONV_F32)
    sh = oracle_shape(cfg)
    check(y, oracle.conv_fwd(sh, x, w), FP32_TOL, "y")
    check(dx, oracle.conv_bwd_data(sh, dy, w), FP32_TOL, "dx")
    check(dw, oracle.conv_bwd_weight(sh, x, dy), FP32_TOL, "dw")
    # and the single-call full layer: same sums, possibly in another order
    check(y, dev.fwd(), SAME_MATH_TOL, "y vs one call")
    check(dx, dev.bwd_data(), SAME_MATH_TOL, "dx vs one call")
    check(dw, dev.bwd_weight(), SAME_MATH_TOL, "dw vs one call")


def test_partitioned_layer_matches_oracle_bf16():
    cfg, times = CASES[1]
    cfg = cfg.with_slice(0, cfg.K)
    x, w, dy = (synth.round_to_bf16(a) for a in synth.make_inputs(cfg))
    _, bounds = cs.conv_partition(times, cfg.K)
    dev = Device(cfg, x, w, dy, dtype=cs.CONV_BF16)
    y, dx, dw = run_layer(dev, cfg, bounds, cs.CONV_BF16)
    sh = oracle_shape(cfg)
    check(y, oracle.conv_fwd(sh, x, w), BF16_TOL, "y")
    check(dx, oracle.conv_bwd_data(sh, dy, w), BF16_TOL, "dx")
    check(dw, oracle.conv_bwd_weight(sh, x, dy), FP32_TOL, "dw")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_large_slices_share_the_input_work_copy(dtype):
    """Slices that each fill the GPU run one after the other on one workspace, and only the first
    re-lays the shared input (Algorithm 1: every device receives the same inputs).  The 1500-kernel
    layer split for four devices against the same layer in one call: the same sums, possibly in
    another order.  (Every element of the one-call result is checked against the oracle elsewhere.)"""
    cfg = synth.CONFIGS["cfg3"]
    x, w, dy = synth.make_inputs(cfg)
    dt = cs.CONV_F32 if dtype == "f32" else cs.CONV_BF16
    if dt == cs.CONV_BF16:
        x, w, dy = (synth.round_to_bf16(a) for a in (x, w, dy))
    _, bounds = cs.conv_partition([0.8, 1.0, 1.7, 2.4], cfg.K)
    dev = Device(cfg, x, w, dy, dtype=dt)
    y, dx, dw = run_layer(dev, cfg, bounds, dt)
    # bf16 tensors differ by at most one rounding of the stored value when the fp32 sums differ in their last bits.
    # dx is the sum of four partial gradients of 9 000 to 14 000 terms each instead of one sum of 37 500 terms:
    # both are fp32 evaluations within the fp32 tolerance of the exact sum, and so is their difference.
    tol = SAME_MATH_TOL if dt == cs.CONV_F32 else 2.0 ** -7
    # (in bf16 every slice's partial gradient is rounded into the bf16 dx as it is added: four roundings instead of one)
    tol_dx = FP32_TOL if dt == cs.CONV_F32 else BF16_TOL
    for got, one, name, t in ((y, dev.fwd(), "y", tol), (dx, dev.bwd_data(), "dx", tol_dx),
                              (dw, dev.bwd_weight(), "dw", SAME_MATH_TOL)):
        e = rel_err(got, one)
        print(f"  {dtype} {name}: partitioned vs one call, rms-floored max rel {e:.3e}; "
              f"{np.count_nonzero(got != one)} of {got.size} elements differ")
        assert e <= t, f"{name}: {e:.3e}"


def test_partitioned_layer_is_bit_stable_and_honours_accumulate():
    cfg, times = CASES[2]
    cfg = cfg.with_slice(0, cfg.K)
    x, w, dy = synth.make_inputs(cfg)
    _, bounds = cs.conv_partition(times, cfg.K)
    dev = Device(cfg, x, w, dy)
    a = run_layer(dev, cfg, bounds, cs.CONV_F32)
    b = run_layer(dev, cfg, bounds, cs.CONV_F32)
    for u, v, name in zip(a, b, ("y", "dx", "dw")):
        assert np.array_equal(u, v), f"{name} differs between two identical calls"
    init = np.full((cfg.N, cfg.C, cfg.H, cfg.W), 1.25, np.float32)
    _, dx, _ = run_layer(dev, cfg, bounds, cs.CONV_F32, dx_init=init, accumulate=1)
    check(dx, oracle.conv_bwd_data(oracle_shape(cfg), dy, w) + 1.25, FP32_TOL, "dx accumulate")


def test_layer_call_orders_with_the_callers_stream():
    """Work enqueued on the caller's stream before and after a conv_layer_* call is ordered
    with the slices that run on the library's own streams."""
    import torch
    cfg, times = CASES[0]
    cfg = cfg.with_slice(0, cfg.K)
    x, w, dy = synth.make_inputs(cfg)
    _, bounds = cs.conv_partition(times, cfg.K)
    dev = Device(cfg, x, w, dy)
    ws = layer_ws(cfg, bounds, cs.CONV_F32)
    ref = oracle.conv_fwd(oracle_shape(cfg), x, w)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        xs = torch.zeros_like(dev.x)
        for _ in range(20):               # a queue of work in front of the input's final value
            xs.add_(1.0)
        xs.copy_(dev.x)
        y = torch.empty((cfg.N, cfg.K, cfg.P, cfg.Q), device="cuda:0")
        cs.conv_layer_fwd(desc_of(cfg), bounds, xs, dev.w, y, ws)
        total = y.double().sum()          # consumer on the caller's stream right after the call
    side.synchronize()
    assert abs(float(total) - ref.sum()) <= 1e-4 * np.abs(ref).sum()
    check(y.cpu().numpy(), ref, FP32_TOL, "y on a side stream")


def test_calibration_probe_reports_a_time_and_scales_with_the_slice():
    import torch
    layer = cs.ConvDesc(128, 64, 28, 28, 256, 3, 3, 1, 1, 1, 1)
    half = cs.ConvDesc(128, 64, 28, 28, 256, 3, 3, 1, 1, 1, 1, 0, 128)
    mask = cs.pass_mask(cs.PASS_FWD, cs.PASS_BWD_DATA, cs.PASS_BWD_WEIGHT)
    ws = torch.empty(cs.conv_calibrate_workspace_bytes(layer, mask), dtype=torch.uint8, device="cuda:0")
    t_full = cs.conv_calibrate(layer, mask, 5, ws)
    t_half = cs.conv_calibrate(half, mask, 5, ws)
    t_fwd = cs.conv_calibrate(layer, 0, 5, ws)
    flops = 3 * 2.0 * 128 * 256 * 64 * 9 * 28 * 28
    assert 1e-5 < t_full < 0.1, t_full
    assert flops / t_full < 157.3e12           # no faster than the fp32 matrix-core peak
    assert t_fwd < t_full                      # forward only is part of the three passes
    assert 0.25 * t_full < t_half < 0.95 * t_full
    # two devices: the GPU itself and a pretend one half as fast -> Eq. (1) gives 2/3, 1/3
    shares, bounds = cs.conv_partition([t_full, 2 * t_full], 256)
    assert shares == pytest.approx([2 / 3, 1 / 3], rel=1e-12)
    assert bounds == [0, 171, 256]
