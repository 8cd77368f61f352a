"""conv_fwd_noalloc (the forward pass on the library's own fixed device array, for callers that
cannot allocate) against conv_fwd with a caller workspace: same kernels, so the results must be
bit-equal; two calls in a row, the second on a smaller layer."""
import numpy as np
import pytest

import oracle
import paper_1712_02546_amd as cs
from helpers import FP32_TOL, Device, desc_of, oracle_shape, rel_err
from paper_1712_02546_amd import synth

pytestmark = pytest.mark.gpu

BIG = synth.random_layer(50, N=40, C=37, H=13, W=11, K=150, R=3, S=5, pad=1, k0=7, k1=141)
SMALL = synth.random_layer(51, N=5, C=8, H=9, W=9, K=12, R=3, S=3, pad=1)


def test_noalloc_forward_equals_workspace_forward_twice_in_a_row():
    import torch
    outs = []
    for cfg in (BIG, SMALL):
        x, w, dy = synth.make_inputs(cfg)
        dev = Device(cfg, x, w, None)
        assert cs.conv_workspace_bytes(desc_of(cfg), cs.PASS_FWD) <= cs.NOALLOC_MAX_WORKSPACE
        y_ws = dev.fwd(fill=3.0)
        y = torch.full((cfg.N, cfg.K, cfg.P, cfg.Q), 3.0, device="cuda:0")
        cs.conv_fwd_noalloc(desc_of(cfg), dev.x, dev.w, y)
        torch.cuda.synchronize()
        y = y.cpu().numpy()
        assert np.array_equal(y, y_ws), f"{cfg.name}: noalloc result differs from the workspace result"
        k0, k1 = cfg.slice
        assert rel_err(y[:, k0:k1], oracle.conv_fwd(oracle_shape(cfg), x, w)[:, k0:k1]) <= FP32_TOL
        outs.append(y)
    # the first layer again after the smaller one: the shared array holds the small call's data now
    x, w, dy = synth.make_inputs(BIG)
    dev = Device(BIG, x, w, None)
    y = torch.full((BIG.N, BIG.K, BIG.P, BIG.Q), 3.0, device="cuda:0")
    cs.conv_fwd_noalloc(desc_of(BIG), dev.x, dev.w, y)
    torch.cuda.synchronize()
    assert np.array_equal(y.cpu().numpy(), outs[0])


def test_noalloc_bf16_and_oversize_refusal():
    import torch
    cfg = synth.random_layer(52, N=33, C=40, H=10, W=10, K=37, R=3, S=3)
    x, w, dy = (synth.round_to_bf16(a) for a in synth.make_inputs(cfg))
    dev = Device(cfg, x, w, None, dtype=cs.CONV_BF16)
    y_ws = dev.fwd(fill=1.0)
    y = torch.full((cfg.N, cfg.K, cfg.P, cfg.Q), 1.0, dtype=torch.bfloat16, device="cuda:0")
    cs.conv_fwd_noalloc(desc_of(cfg, cs.CONV_BF16), dev.x, dev.w, y)
    torch.cuda.synchronize()
    assert np.array_equal(y.float().cpu().numpy(), y_ws)
    big = synth.CONFIGS["cfg3"]
    assert cs.conv_workspace_bytes(desc_of(big), cs.PASS_FWD) > cs.NOALLOC_MAX_WORKSPACE
    assert cs.conv_fwd_noalloc(desc_of(big), dev.x, dev.w, y, raw_status=True) == -5
