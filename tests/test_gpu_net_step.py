"""One training step of the paper's network (Section 4.1's layer list) through the library
against the same step composed from the oracles: loss, every gradient, and the updated weights."""
import numpy as np
import pytest

import oracle
from helpers import rel_err
from oracle import netlayers as on
from paper_1712_02546_amd import net as pnet

pytestmark = pytest.mark.gpu


def oracle_step(x, labels, w1, w2, wf, bf, lr):
    N, K1, K2 = x.shape[0], w1.shape[0], w2.shape[0]
    s1 = oracle.Shape(N, 3, 32, 32, K1, 5, 5, 1, 1, 0, 0, 0, K1)
    s2 = oracle.Shape(N, K1, 14, 14, K2, 5, 5, 1, 1, 0, 0, 0, K2)
    a1 = oracle.conv_fwd(s1, x, w1)
    n1 = on.norm_fwd(a1, **pnet.NORM)
    p1 = on.pool_fwd(n1)
    a2 = oracle.conv_fwd(s2, p1, w2)
    n2 = on.norm_fwd(a2, **pnet.NORM)
    p2 = on.pool_fwd(n2)
    z = on.fc_fwd(p2, wf, bf)
    loss = on.softmax_loss_fwd(z, labels)
    gz = on.softmax_loss_bwd(z, labels)
    gp2, gwf, gbf = on.fc_bwd(p2, wf, gz)
    gn2 = on.pool_bwd(n2, gp2)
    ga2 = on.norm_bwd(a2, gn2, **pnet.NORM)
    gw2 = oracle.conv_bwd_weight(s2, p1, ga2)
    gp1 = oracle.conv_bwd_data(s2, ga2, w2)
    gn1 = on.pool_bwd(n1, gp1)
    ga1 = on.norm_bwd(a1, gn1, **pnet.NORM)
    gw1 = oracle.conv_bwd_weight(s1, x, ga1)
    return dict(loss=loss, gw1=gw1, gw2=gw2, gwf=gwf, gbf=gbf, gp1=gp1,
                w1=on.sgd_update(w1, gw1, lr), w2=on.sgd_update(w2, gw2, lr), wf=on.sgd_update(wf, gwf, lr))


@pytest.mark.parametrize("N,K1,K2", [(4, 6, 8), (33, 20, 40)])
def test_training_step_matches_the_oracles(N, K1, K2):
    import torch
    net = pnet.PaperNet(N, K1, K2, seed=5, lr=0.05)
    rng = np.random.default_rng(N)
    x = rng.random((N, 3, 32, 32)).astype(np.float32)
    labels = rng.integers(0, 10, size=N).astype(np.int32)
    w1, w2, wf, bf = (t.double().cpu().numpy() for t in (net.w1, net.w2, net.wf, net.bf))
    ref = oracle_step(x.astype(np.float64), labels, w1, w2, wf, bf, float(np.float32(0.05)))
    net.step(torch.from_numpy(x).cuda(), torch.from_numpy(labels).cuda())
    conv_ms, other_ms = net.times_ms()
    assert conv_ms > 0 and other_ms > 0
    got = {k: getattr(net, k).double().cpu().numpy() for k in ("gw1", "gw2", "gwf", "gbf", "gp1", "w1", "w2", "wf")}
    assert abs(float(net.loss.cpu()[0]) - ref["loss"]) <= 1e-5 * abs(ref["loss"])
    # a chain of fp32 layers: the tolerance of one layer, times a small factor for the depth
    for k, v in got.items():
        assert rel_err(v, ref[k]) <= 3e-4, k
