"""HIP path vs CPU oracle, element by element, on the same seeded inputs (needs an MI355X)."""
import numpy as np
import pytest

import oracle
import paper_1712_02546_amd as cs
from paper_1712_02546_amd import synth

from helpers import BF16_TOL, FP32_TOL, Device, desc_of, oracle_shape, rel_err, sample_indices

pytestmark = pytest.mark.gpu

# Small enough for the full oracle in seconds, large enough for several 128-wide tiles,
# ragged tails in every GEMM dimension, batches that are not multiples of 32, strides,
# padding, rectangular filters and interior slices.
ADHOC = [
    synth.random_layer(1, N=40, C=37, H=13, W=11, K=150, R=3, S=5),
    synth.random_layer(2, N=40, C=37, H=13, W=11, K=150, R=3, S=5, stride=2, pad=2, k0=7, k1=141),
    synth.random_layer(3, N=5, C=8, H=9, W=9, K=12, R=3, S=3, pad=1),
    synth.random_layer(4, N=130, C=140, H=8, W=8, K=20, R=3, S=3, pad=1, k0=3, k1=20),
    synth.random_layer(5, N=33, C=3, H=23, W=19, K=70, R=7, S=4, stride=3, pad=3),
    synth.random_layer(6, N=64, C=16, H=6, W=6, K=300, R=6, S=6, k0=100, k1=290),      # P = Q = 1
    synth.random_layer(7, N=32, C=20, H=10, W=10, K=33, R=1, S=1),                    # 1x1
    synth.random_layer(8, N=9, C=5, H=34, W=34, K=6, R=5, S=5, stride=4),             # unread last row/col
    synth.random_layer(9, N=1, C=1, H=5, W=5, K=1, R=2, S=2),
    # more than 512 tiles with a long reduction: the tail tiles are shared out in runs
    synth.random_layer(10, N=32, C=64, H=34, W=34, K=200, R=3, S=3, k0=9, k1=200),
    synth.random_layer(11, N=3, C=2, H=33, W=34, K=3, R=32, S=32),                   # R*S at the limit
    synth.random_layer(12, N=65, C=32, H=9, W=7, K=70, R=3, S=2, stride=2, pad=1),    # bf16: C = 32, batch 65
    synth.random_layer(13, N=20, C=72, H=10, W=10, K=130, R=5, S=5, pad=2, k0=1, k1=130),
    # input-gradient tiles of unequal length shared out in equal runs (batch fills whole column tiles)
    synth.random_layer(14, N=128, C=130, H=12, W=12, K=100, R=3, S=3, pad=1, k0=2, k1=100),
    # the same with pixels no tap reaches (1x1, stride 2)
    synth.random_layer(15, N=100, C=130, H=24, W=24, K=260, R=1, S=1, stride=2),
    # column tiles that span pixels with different tap sets (three image blocks per pixel, stride 2)
    synth.random_layer(16, N=70, C=100, H=9, W=11, K=40, R=3, S=3, stride=2, pad=1, k0=0, k1=37),
    # filters longer than 32 taps along an axis, with enough channels for the per-pixel input-gradient form
    synth.random_layer(17, N=2, C=64, H=40, W=10, K=8, R=33, S=3),
    synth.random_layer(18, N=2, C=40, H=34, W=34, K=4, R=32, S=32),                  # R*S at the limit, per pixel
    synth.random_layer(19, N=3, C=48, H=70, W=5, K=5, R=64, S=2, stride=2, pad=1),
    # few input channels (pixel-major path): odd P*Q, padding and stride, a full plus a half row tile
    synth.random_layer(22, N=3, C=3, H=20, W=17, K=190, R=5, S=3, stride=2, pad=1),
    # P*Q a multiple of 4, interior slice of 132 kernels, 36 taps (half row tile in the input gradient), ragged columns
    synth.random_layer(23, N=6, C=4, H=16, W=16, K=140, R=3, S=3, k0=5, k1=137),
    # C*R*S = 480, the most the pixel-major path takes; 8.75 reduction chunks per image in the weight gradient
    synth.random_layer(24, N=2, C=16, H=12, W=40, K=33, R=5, S=6),
    # bf16: more 256 x 256 tiles than compute units (whole tiles plus a shared tail), a ragged second row tile of
    # 31 kernels, 162 channels (ragged second row tile of the input gradient), padding
    synth.random_layer(25, N=40, C=162, H=24, W=24, K=300, R=3, S=3, pad=1, k0=3, k1=290),
    # a full row tile plus a 96-row tile with ragged rows in every pass: 210 = 128 + 82 channels, 215 = 128 + 87 kernels
    synth.random_layer(26, N=33, C=210, H=9, W=9, K=215, R=3, S=3, pad=1),
    # only a 96-row tile, stride 2, batch of one block: 90 channels, 70 kernels
    synth.random_layer(27, N=20, C=90, H=11, W=10, K=70, R=3, S=2, stride=2),
    # 1 200 forward tiles of 18 chunks for 512 workgroup slots: two rounds of whole tiles, 176 tiles shared in runs of
    # 7 chunks; 36 weight-gradient tiles of 2 400 chunks, the reduction split
    synth.random_layer(30, N=32, C=64, H=48, W=50, K=260, R=3, S=3, pad=1, k0=2, k1=258),
    # bf16: 17 channels (a quarter of a 64-channel chunk, 17 of an input-gradient tile's 128 rows), and 8 channels with
    # C*R*S = 512, just past what the few-channel path takes
    synth.random_layer(31, N=20, C=17, H=12, W=11, K=70, R=3, S=3, pad=1, k0=3, k1=70),
    synth.random_layer(32, N=9, C=8, H=14, W=13, K=40, R=8, S=8, pad=2),
    # few channels, one filter row with stride 4: three of four rows of dx are reached by no tap, the rest by one or two
    synth.random_layer(28, N=100, C=12, H=15, W=19, K=288, R=1, S=5, stride=4, pad=3, k0=29, k1=122),
]


# Two correct fp32 evaluations of the same sums in different orders (error metric of helpers.rel_err).
SAME_MATH_TOL = 2e-5


def check(got, ref, tol, what):
    e = rel_err(got, ref)
    assert e <= tol, f"{what}: max rel err {e:.3e} > {tol:.1e}"


@pytest.mark.parametrize("cfg", ADHOC + [synth.CONFIGS["cfg1"]], ids=lambda c: c.name)
def test_full_tensors_match_oracle_fp32(cfg):
    x, w, dy = synth.make_inputs(cfg)
    sh = oracle_shape(cfg)
    k0, k1 = cfg.slice
    dev = Device(cfg, x, w, dy)
    y = dev.fwd(fill=7.0)
    y_ref = oracle.conv_fwd(sh, x, w)
    check(y[:, k0:k1], y_ref[:, k0:k1], FP32_TOL, "y")
    assert np.all(y[:, :k0] == 7.0) and np.all(y[:, k1:] == 7.0), "channels outside the slice were written"
    dx = dev.bwd_data()
    check(dx, oracle.conv_bwd_data(sh, dy, w), FP32_TOL, "dx")
    dw = dev.bwd_weight(fill=7.0)
    dw_ref = oracle.conv_bwd_weight(sh, x, dy)
    check(dw[k0:k1], dw_ref[k0:k1], FP32_TOL, "dw")
    assert np.all(dw[:k0] == 7.0) and np.all(dw[k1:] == 7.0), "filters outside the slice were written"


@pytest.mark.parametrize("cfg", [ADHOC[1], ADHOC[3], ADHOC[4], ADHOC[7], ADHOC[11], ADHOC[12], ADHOC[13], ADHOC[16], ADHOC[19],
                          ADHOC[20], ADHOC[21], ADHOC[22], synth.CONFIGS["cfg1"]]
                         # 17 and 8 channels on the bf16 matrix cores; P*Q = 1 with 16 channels; and the two cases that still
                         # multiply in fp32 (fewer than 8 channels outside the few-channel path: P*Q = 16, C*R*S = 2048)
                         + [c for c in ADHOC if c.name in ("adhoc31", "adhoc32", "adhoc6", "adhoc9", "adhoc11")],
                         ids=lambda c: c.name)
def test_full_tensors_match_oracle_bf16(cfg):
    xo, wo, dyo = synth.make_inputs(cfg)
    x, w, dy = (synth.round_to_bf16(a) for a in (xo, wo, dyo))
    sh = oracle_shape(cfg)
    k0, k1 = cfg.slice
    dev = Device(cfg, x, w, dy, dtype=cs.CONV_BF16)
    y, dx, dw = dev.fwd(), dev.bwd_data(), dev.bwd_weight()
    # against the oracle on the rounded inputs: accumulation and output rounding only
    check(y[:, k0:k1], oracle.conv_fwd(sh, x, w)[:, k0:k1], BF16_TOL, "y")
    check(dx, oracle.conv_bwd_data(sh, dy, w), BF16_TOL, "dx")
    # dw is stored in fp32, so it is held to the fp32 tolerance on the rounded inputs
    check(dw[k0:k1], oracle.conv_bwd_weight(sh, x, dy)[k0:k1], FP32_TOL, "dw")
    # against the oracle on the inputs before rounding: input rounding included
    check(y[:, k0:k1], oracle.conv_fwd(sh, xo, wo)[:, k0:k1], BF16_TOL, "y vs unrounded inputs")
    check(dx, oracle.conv_bwd_data(sh, dyo, wo), BF16_TOL, "dx vs unrounded inputs")
    check(dw[k0:k1], oracle.conv_bwd_weight(sh, xo, dyo)[k0:k1], BF16_TOL, "dw vs unrounded inputs")


def test_wide_input_gradient_tiles_one_workgroup_each_bf16():
    """More 256 x 256 input-gradient tiles than compute units (no runs: one workgroup per tile, heaviest first),
    with pixels that no tap reaches (1x1, stride 2).  Compared on the rounded inputs only: with one tap and 260
    kernels per sum, the rounding of the inputs alone moves single elements of dx by 2.3 % of the tensor's rms,
    whatever kernel adds them up; the gate on unrounded inputs is held by the cases above."""
    cfg = ADHOC[14]
    x, w, dy = (synth.round_to_bf16(a) for a in synth.make_inputs(cfg))
    sh = oracle_shape(cfg)
    dev = Device(cfg, x, w, dy, dtype=cs.CONV_BF16)
    assert "wide" in cs.conv_pass_path(desc_of(cfg, cs.CONV_BF16), cs.PASS_BWD_DATA)
    check(dev.fwd(), oracle.conv_fwd(sh, x, w), BF16_TOL, "y")
    check(dev.bwd_data(), oracle.conv_bwd_data(sh, dy, w), BF16_TOL, "dx")
    check(dev.bwd_weight(), oracle.conv_bwd_weight(sh, x, dy), FP32_TOL, "dw")


def test_few_channel_input_gradient_keeps_fp32_sums_bf16():
    """bf16 input gradient of a few-channel layer (T = w^T dy on the bf16 matrix cores, then the sum over taps) where
    three quarters of dx are zero by construction, so the error metric's rms floor is low and taps that cancel
    show: the sums over kernels must reach the sum over taps unrounded (T in fp32), or single elements miss the
    tolerance.  Rounded inputs only, for the reason given in the test above."""
    cfg = next(c for c in ADHOC if c.name == "adhoc28")
    x, w, dy = (synth.round_to_bf16(a) for a in synth.make_inputs(cfg))
    sh = oracle_shape(cfg)
    k0, k1 = cfg.slice
    dev = Device(cfg, x, w, dy, dtype=cs.CONV_BF16)
    assert cs.conv_pass_path(desc_of(cfg, cs.CONV_BF16), cs.PASS_BWD_DATA).startswith("bwd_data16_pm_gemm_kernel")
    check(dev.fwd()[:, k0:k1], oracle.conv_fwd(sh, x, w)[:, k0:k1], BF16_TOL, "y")
    check(dev.bwd_data(), oracle.conv_bwd_data(sh, dy, w), BF16_TOL, "dx")
    check(dev.bwd_weight()[k0:k1], oracle.conv_bwd_weight(sh, x, dy)[k0:k1], FP32_TOL, "dw")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_few_channel_input_gradient_in_image_groups(dtype):
    """T = w^T dy of this layer is 169 MiB (13 images x 363 taps x 97 x 97 pixels), above the size up to which it is
    computed in one pass: the images go through in groups of 7 and 6, on top of an initial dx (accumulate)."""
    cfg = synth.random_layer(29, N=13, C=3, H=200, W=200, K=16, R=11, S=11, stride=2, pad=2, k0=1, k1=15)
    bf = dtype == "bf16"
    x, w, dy = synth.make_inputs(cfg)
    if bf:
        x, w, dy = (synth.round_to_bf16(a) for a in (x, w, dy))
    init = np.random.default_rng(5).standard_normal((cfg.N, cfg.C, cfg.H, cfg.W)).astype(np.float32)
    if bf:
        init = synth.round_to_bf16(init)
    dev = Device(cfg, x, w, dy, dtype=cs.CONV_BF16 if bf else cs.CONV_F32)
    assert "pm_gemm_kernel" in cs.conv_pass_path(desc_of(cfg, dev.dtype), cs.PASS_BWD_DATA)
    ref = oracle.conv_bwd_data(oracle_shape(cfg), dy, w)
    tol = BF16_TOL if bf else FP32_TOL
    check(dev.bwd_data(), ref, tol, "dx")
    check(dev.bwd_data(accumulate=1, init=init), ref + init, tol, "dx on top of an initial value")


@pytest.mark.parametrize("C", [24, 48])
def test_disjoint_slices_assemble_the_full_layer(C):
    """Same inputs, different kernels per device, outputs side by side (Section 4.1.2):
    slice calls into one y / dw give the full result; dx partial sums add up."""
    import torch
    cfg = synth.random_layer(20, N=36, C=C, H=12, W=12, K=200, R=5, S=5, pad=1)
    x, w, dy = synth.make_inputs(cfg)
    full = Device(cfg, x, w, dy)
    y_full, dw_full, dx_full = full.fwd(), full.bwd_weight(), full.bwd_data()
    y = torch.zeros((cfg.N, cfg.K, cfg.P, cfg.Q), device="cuda:0")
    dw = torch.zeros((cfg.K, cfg.C, cfg.R, cfg.S), device="cuda:0")
    dx = torch.empty((cfg.N, cfg.C, cfg.H, cfg.W), device="cuda:0")
    cuts = [0, 37, 37, 128, 200]
    from helpers import desc_of
    for i, (k0, k1) in enumerate(zip(cuts[:-1], cuts[1:])):
        part = cfg.with_slice(k0, k1)
        cs.conv_fwd(desc_of(part), full.x, full.w, y, full.ws)
        cs.conv_bwd_weight(desc_of(part), full.x, full.dy, dw, full.ws)
        cs.conv_bwd_data(desc_of(part, accumulate=int(i > 0)), full.dy, full.w, dx, full.ws)
    torch.cuda.synchronize()
    # The split of a reduction over workgroups depends on how many tiles a call has, so a slice
    # call and the full-layer call may round differently: equal up to fp32 summation order.
    check(y.cpu().numpy(), y_full, SAME_MATH_TOL, "y assembled")
    check(dw.cpu().numpy(), dw_full, SAME_MATH_TOL, "dw assembled")
    check(dx.cpu().numpy(), dx_full, SAME_MATH_TOL, "dx summed")
    check(dx.cpu().numpy(), oracle.conv_bwd_data(oracle_shape(cfg), dy, w), FP32_TOL, "dx vs oracle")


@pytest.mark.parametrize("C", [6, 40])   # few channels: scatter form; many: per-pixel form
def test_empty_slice_and_accumulate(C):
    cfg = synth.random_layer(21, N=7, C=C, H=9, W=9, K=10, R=3, S=3, k0=4, k1=4)
    x, w, dy = synth.make_inputs(cfg)
    dev = Device(cfg, x, w, dy)
    assert np.all(dev.fwd(fill=3.0) == 3.0)
    assert np.all(dev.bwd_weight(fill=3.0) == 3.0)
    assert not dev.bwd_data().any()
    init = np.full((cfg.N, cfg.C, cfg.H, cfg.W), 2.5, np.float32)
    assert np.all(dev.bwd_data(accumulate=1, init=init) == 2.5)
    cfg2 = cfg.with_slice(2, 9)
    dev2 = Device(cfg2, x, w, dy)
    ref = oracle.conv_bwd_data(oracle_shape(cfg2), dy, w)
    check(dev2.bwd_data(accumulate=1, init=init), ref + 2.5, FP32_TOL, "dx accumulate")


@pytest.mark.parametrize("which,dtype", [(1, "f32"), (9, "f32"), (14, "f32"), (12, "bf16")])
def test_results_are_bit_stable_run_to_run(which, dtype):
    """No atomics anywhere: split reductions and shared tails are summed in a fixed order."""
    cfg = ADHOC[which]
    x, w, dy = synth.make_inputs(cfg)
    dev = Device(cfg, x, w, dy, dtype=cs.CONV_F32 if dtype == "f32" else cs.CONV_BF16)
    a = (dev.fwd(fill=0.0), dev.bwd_data(), dev.bwd_weight(fill=0.0))
    b = (dev.fwd(fill=0.0), dev.bwd_data(), dev.bwd_weight(fill=0.0))
    for u, v in zip(a, b):
        assert np.array_equal(u, v)


# ------------------------------------------------ full benchmark sizes, every element
# The oracle computes the whole layer of a seed family once (all K kernels); configurations
# that are slices of it (the device share, the eighth shares) compare against its channels.
# Two families are kept, so that consecutive tests on one family do not recompute it.
_FULL = {}


def _full_layer_oracle(cfg, rounded):
    """(x, w, dy, y_ref, dw_ref) for all K kernels of cfg's layer; inputs rounded to bf16 first if asked."""
    key = (cfg.index, cfg.N, cfg.C, cfg.H, cfg.W, cfg.K, cfg.R, cfg.S, cfg.stride, cfg.pad, rounded)
    if key not in _FULL:
        while len(_FULL) >= 2:
            _FULL.pop(next(iter(_FULL)))
        whole = cfg.with_slice(0, cfg.K)
        x, w, dy = synth.make_inputs(whole)
        if rounded:
            x, w, dy = (synth.round_to_bf16(a) for a in (x, w, dy))
        sh = oracle_shape(whole)
        _FULL[key] = (x, w, dy, oracle.conv_fwd(sh, x, w), oracle.conv_bwd_weight(sh, x, dy))
    else:
        _FULL[key] = _FULL.pop(key)   # most recently used last
    return _FULL[key]


def _report(what, got, ref, tol):
    """Gate on the declared metric (RMS-floored relative error); print the two plain figures beside it."""
    got = np.asarray(got, dtype=np.float64)
    e = rel_err(got, ref)
    diff = np.abs(got - ref)
    inf_ratio = float(diff.max() / np.abs(ref).max())
    big = np.abs(ref) >= 1e-3 * np.abs(ref).max()          # plain relative error where the reference is not tiny
    plain = float((diff[big] / np.abs(ref[big])).max())
    print(f"  {what}: rms-floored max rel {e:.3e} (gate {tol:.0e}); |g-o|_inf/|o|_inf {inf_ratio:.3e}; "
          f"plain max rel over |o| >= 1e-3 |o|_inf {plain:.3e}")
    assert e <= tol, f"{what}: max rel err {e:.3e} > {tol:.1e}"


def _full(cfg, dtype):
    """All three passes at full size against the oracle, every element of the slice."""
    k0, k1 = cfg.slice
    bf16 = dtype == cs.CONV_BF16
    x, w, dy, y_ref, dw_ref = _full_layer_oracle(cfg, rounded=bf16)
    sh = oracle_shape(cfg)
    dev = Device(cfg, x, w, dy, dtype=dtype)
    tag = f"{cfg.name}[{k0},{k1}) {'bf16' if bf16 else 'f32'}"
    tol = BF16_TOL if bf16 else FP32_TOL
    y = dev.fwd(fill=5.0)
    _report(f"{tag} y", y[:, k0:k1], y_ref[:, k0:k1], tol)
    if k0 > 0 or k1 < cfg.K:
        assert np.all(y[:, :k0] == 5.0) and np.all(y[:, k1:] == 5.0), "channels outside the slice were written"
    dx = dev.bwd_data()
    dx_ref = oracle.conv_bwd_data(sh, dy, w)
    _report(f"{tag} dx", dx, dx_ref, tol)
    dw = dev.bwd_weight(fill=5.0)
    _report(f"{tag} dw", dw[k0:k1], dw_ref[k0:k1], FP32_TOL)   # dw is fp32 also on the bf16 path
    if k0 > 0 or k1 < cfg.K:
        assert np.all(dw[:k0] == 5.0) and np.all(dw[k1:] == 5.0), "filters outside the slice were written"
    if not bf16:
        return
    # The same device results against the oracle on the inputs BEFORE rounding to bf16: input
    # rounding, accumulation and output rounding together must stay inside the bf16 tolerance.
    xo, wo, dyo, yo_ref, dwo_ref = _full_layer_oracle(cfg, rounded=False)
    _report(f"{tag} y vs oracle on unrounded inputs", y[:, k0:k1], yo_ref[:, k0:k1], BF16_TOL)
    _report(f"{tag} dx vs oracle on unrounded inputs", dx, oracle.conv_bwd_data(sh, dyo, wo), BF16_TOL)
    _report(f"{tag} dw vs oracle on unrounded inputs", dw[k0:k1], dwo_ref[k0:k1], BF16_TOL)


FULL_SIZE = [("cfg2", "f32"), ("cfg5a", "f32"), ("cfg5a", "bf16"), ("cfg5b", "f32"), ("cfg5b", "bf16"),
             ("cfg3", "f32"), ("cfg4", "f32")]


@pytest.mark.parametrize("name,dtype", FULL_SIZE)
def test_benchmark_configs_every_element(name, dtype):
    _full(synth.CONFIGS[name], cs.CONV_F32 if dtype == "f32" else cs.CONV_BF16)


@pytest.mark.parametrize("k0,k1", [(188, 376), (1313, 1500), (0, 64)])
def test_eighth_of_the_large_layer_every_element_fp32(k0, k1):
    """One of eight equal shares of the 1500-kernel layer (Eq. (1) with equal devices): two
    96-row tiles in the forward and weight-gradient passes; and a share that is a 64-row tile
    only."""
    _full(synth.CONFIGS["cfg3"].with_slice(k0, k1), cs.CONV_F32)


def test_large_layer_every_element_bf16():
    _full(synth.CONFIGS["cfg3"], cs.CONV_BF16)


def test_device_share_of_the_large_layer_every_element_bf16():
    """Kernels 500..999: 256 x 256 tiles in the forward and weight-gradient passes (the latter in equal runs),
    128 x 128 tiles in the input gradient, whose runs would be short."""
    _full(synth.CONFIGS["cfg4"], cs.CONV_BF16)


def test_full_size_oracle_cache_is_released():
    _FULL.clear()


def _sampled(cfg, dtype, tol, n=1500):
    """Sampled comparison, for layers too large for the full oracle."""
    x, w, dy = synth.make_inputs(cfg)
    if dtype == cs.CONV_BF16:
        x, w, dy = (synth.round_to_bf16(a) for a in (x, w, dy))
    sh = oracle_shape(cfg)
    k0, k1 = cfg.slice
    dev = Device(cfg, x, w, dy, dtype=dtype)
    # forward: sample inside the slice
    y = dev.fwd(fill=5.0)
    ysl = y[:, k0:k1]
    idx = sample_indices(ysl.size, n, 1)
    nn, kk, pp, qq = np.unravel_index(idx, ysl.shape)
    flat = np.ravel_multi_index((nn, kk + k0, pp, qq), y.shape)
    ref = oracle.conv_fwd_at(sh, x, w, flat)
    scale = float(np.sqrt(np.mean(ref * ref)))
    err = np.max(np.abs(y.ravel()[flat] - ref) / np.maximum(np.abs(ref), scale))
    assert err <= tol, f"y sampled: {err:.3e}"
    if k0 > 0 or k1 < cfg.K:
        assert np.all(y[:, :k0] == 5.0) and np.all(y[:, k1:] == 5.0)
    del y, ysl
    dx = dev.bwd_data()
    idx = sample_indices(dx.size, n, 2)
    ref = oracle.conv_bwd_data_at(sh, dy, w, idx)
    scale = float(np.sqrt(np.mean(ref * ref)))
    err = np.max(np.abs(dx.ravel()[idx] - ref) / np.maximum(np.abs(ref), scale))
    assert err <= tol, f"dx sampled: {err:.3e}"
    del dx
    dw = dev.bwd_weight(fill=5.0)
    dwsl = dw[k0:k1]
    idx = sample_indices(dwsl.size, n, 3)
    flat = idx + k0 * cfg.C * cfg.R * cfg.S
    ref = oracle.conv_bwd_weight_at(sh, x, dy, flat)
    scale = float(np.sqrt(np.mean(ref * ref)))
    err = np.max(np.abs(dw.ravel()[flat] - ref) / np.maximum(np.abs(ref), scale))
    assert err <= (tol if dtype == cs.CONV_F32 else FP32_TOL), f"dw sampled: {err:.3e}"
    if k0 > 0 or k1 < cfg.K:
        assert np.all(dw[:k0] == 5.0) and np.all(dw[k1:] == 5.0)


def test_device_share_equals_slice_of_full_layer():
    """cfg4 is kernels 500..999 of cfg3: its maps must be the matching channels of the
    full-layer forward result (up to fp32 summation order) and nothing else is written."""
    full, part = synth.CONFIGS["cfg3"], synth.CONFIGS["cfg4"]
    x, w, dy = synth.make_inputs(full)
    d_full = Device(full, x, w, dy)
    y_full = d_full.fwd()
    d_part = Device(part, None, None, None)
    d_part.x, d_part.w, d_part.dy = d_full.x, d_full.w, d_full.dy
    y_part = d_part.fwd(fill=0.0)
    check(y_part[:, 500:1000], y_full[:, 500:1000], SAME_MATH_TOL, "share vs full layer")
    assert not y_part[:, :500].any() and not y_part[:, 1000:].any()


def test_work_copies_beyond_two_gibibytes_fp32():
    """A layer whose transposed input (and input gradient) is 2 GiB: byte offsets inside the
    work copies pass 2^31, which the 32-bit lane offsets and 64-bit bases of the DMA loads
    must handle.  Sampled against the oracle (the oracle's sampled routines work element by element)."""
    cfg = synth.random_layer(40, N=256, C=512, H=64, W=64, K=8, R=3, S=3, k0=1, k1=8)
    assert cfg.N * cfg.C * cfg.H * cfg.W * 4 == 1 << 31
    _sampled(cfg, cs.CONV_F32, FP32_TOL, n=400)
