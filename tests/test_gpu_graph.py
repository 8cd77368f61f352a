"""The three passes recorded into a HIP graph and replayed: the entry points only launch kernels on the caller's
stream (no allocation, no synchronisation, no memset node), so a launch-bound step of a small layer can be
replayed as one graph.  Every replay must reproduce the eager results bit for bit."""
import numpy as np
import pytest

import paper_1712_02546_amd as cs
from helpers import Device, desc_of
from paper_1712_02546_amd import synth

pytestmark = pytest.mark.gpu

CASES = [
    synth.CONFIGS["cfg1"],                                                                      # few-channel kernels
    synth.random_layer(2, N=40, C=37, H=13, W=11, K=150, R=3, S=5, stride=2, pad=2, k0=7, k1=141),   # shared tails, a slice
]


@pytest.mark.parametrize("cfg", CASES, ids=lambda c: c.name)
@pytest.mark.parametrize("dtype", [cs.CONV_F32, cs.CONV_BF16], ids=["f32", "bf16"])
def test_step_replays_from_a_graph(cfg, dtype):
    import torch
    x, w, dy = synth.make_inputs(cfg)
    if dtype == cs.CONV_BF16:
        x, w, dy = (synth.round_to_bf16(a) for a in (x, w, dy))
    dev = Device(cfg, x, w, dy, dtype=dtype)
    d = desc_of(cfg, dtype)

    def outputs():
        return (dev._empty((cfg.N, cfg.K, cfg.P, cfg.Q), fill=0.0), dev._empty((cfg.N, cfg.C, cfg.H, cfg.W), fill=0.0),
                dev._empty((cfg.K, cfg.C, cfg.R, cfg.S), fp32=True, fill=0.0))

    def step(y, dx, dw):
        cs.conv_fwd(d, dev.x, dev.w, y, dev.ws)
        cs.conv_bwd_data(d, dev.dy, dev.w, dx, dev.ws)
        cs.conv_bwd_weight(d, dev.x, dev.dy, dw, dev.ws)

    eager = outputs()
    step(*eager)          # also the warm-up that sets the kernels' attributes before anything is recorded
    torch.cuda.synchronize()
    want = [t.float().cpu().numpy() for t in eager]

    out = outputs()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(*out)        # the binding takes torch's current stream: the one being recorded
    for replay in range(3):
        for t in out:
            t.zero_()     # the program's own eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, t, ref in zip(("y", "dx", "dw"), out, want):
            assert np.array_equal(t.float().cpu().numpy(), ref), f"replay {replay}: {name} differs from the eager call"
