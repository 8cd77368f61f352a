"""The paper's network (arXiv 1712.02546, Section 4.1) as a sequence of library calls:
C1 5x5 -> normalisation -> pooling /2 -> C2 5x5 -> normalisation -> pooling /2 -> fully
connected -> softmax loss, forward, backward and a plain gradient step.  Every operation runs
in the library's kernels; this file only owns the buffers and the order of the calls, and keeps
per-call HIP event pairs so that the time in convolutions ("Conv. time") and in the other
layers ("Comp. time", Section 4.2) can be read separately.

Input 3 x 32 x 32 (CIFAR-shaped), ten classes; the convolutions have no padding and stride 1
(32 -> 28 -> 14 -> 10 -> 5), as the paper's Eq. (2) extents imply.
"""
from __future__ import annotations

from . import binding as cs

CLASSES = 10
NORM = dict(size=5, kappa=1.0, alpha=1e-4, beta=0.75)


class PaperNet:
    def __init__(self, batch: int, k1: int, k2: int, seed: int = 0, lr: float = 0.01):
        import torch
        self.torch = torch
        self.N, self.K1, self.K2, self.lr = batch, k1, k2, lr
        dev = torch.device("cuda:0")
        g = torch.Generator(device="cpu").manual_seed(seed)

        def rnd(shape, std):
            return (torch.randn(shape, generator=g) * std).to(dev)

        N = batch
        self.w1 = rnd((k1, 3, 5, 5), 0.05)
        self.w2 = rnd((k2, k1, 5, 5), 0.01)
        self.I = k2 * 5 * 5
        self.wf = rnd((CLASSES, self.I), 0.01)
        self.bf = torch.zeros(CLASSES, device=dev)
        self.d1 = cs.ConvDesc(N, 3, 32, 32, k1, 5, 5)
        self.d2 = cs.ConvDesc(N, k1, 14, 14, k2, 5, 5)
        e = lambda *s: torch.empty(s, device=dev)   # noqa: E731
        self.a1, self.n1, self.s1, self.p1 = e(N, k1, 28, 28), e(N, k1, 28, 28), e(N, k1, 28, 28), e(N, k1, 14, 14)
        self.a2, self.n2, self.s2, self.p2 = e(N, k2, 10, 10), e(N, k2, 10, 10), e(N, k2, 10, 10), e(N, k2, 5, 5)
        self.z, self.loss = e(N, CLASSES), e(1)
        # gradients (named after the tensor they belong to)
        self.gz, self.gp2, self.gn2, self.ga2 = e(N, CLASSES), e(N, k2, 5, 5), e(N, k2, 10, 10), e(N, k2, 10, 10)
        self.gp1, self.gn1, self.ga1 = e(N, k1, 14, 14), e(N, k1, 28, 28), e(N, k1, 28, 28)
        self.gw1, self.gw2 = torch.empty_like(self.w1), torch.empty_like(self.w2)
        self.gwf, self.gbf = torch.empty_like(self.wf), torch.empty_like(self.bf)
        need = max(cs.conv_workspace_bytes(d, p) for d in (self.d1, self.d2) for p in (0, 1, 2))
        self.ws = torch.empty(need, dtype=torch.uint8, device=dev)
        self.timeline = []   # (kind, start event, stop event) of the last step, kind in {"conv", "other"}

    def _timed(self, kind, fn, *args, **kw):
        t = self.torch
        a, b = t.cuda.Event(enable_timing=True), t.cuda.Event(enable_timing=True)
        a.record()
        fn(*args, **kw)
        b.record()
        self.timeline.append((kind, a, b))

    def step(self, x, labels, update: bool = True):
        """One training step on images x [N,3,32,32] (fp32) and int32 labels; returns nothing (the
        loss stays in self.loss on the device)."""
        N, K1, K2 = self.N, self.K1, self.K2
        T = self._timed
        self.timeline = []
        # forward
        T("conv", cs.conv_fwd, self.d1, x, self.w1, self.a1, self.ws)
        T("other", cs.net_norm_fwd, self.a1, self.n1, self.s1, N, K1, 28 * 28, **NORM)
        T("other", cs.net_pool_fwd, self.n1, self.p1, N * K1, 28, 28)
        T("conv", cs.conv_fwd, self.d2, self.p1, self.w2, self.a2, self.ws)
        T("other", cs.net_norm_fwd, self.a2, self.n2, self.s2, N, K2, 10 * 10, **NORM)
        T("other", cs.net_pool_fwd, self.n2, self.p2, N * K2, 10, 10)
        T("other", cs.net_fc_fwd, self.p2, self.wf, self.bf, self.z, N, self.I, CLASSES)
        T("other", cs.net_softmax_loss_fwd, self.z, labels, self.loss, N, CLASSES)
        # backward
        T("other", cs.net_softmax_loss_bwd, self.z, labels, self.gz, N, CLASSES)
        T("other", cs.net_fc_bwd, self.p2, self.wf, self.gz, self.gp2, self.gwf, self.gbf, N, self.I, CLASSES)
        T("other", cs.net_pool_bwd, self.n2, self.gp2, self.gn2, N * K2, 10, 10)
        T("other", cs.net_norm_bwd, self.a2, self.n2, self.s2, self.gn2, self.ga2, N, K2, 10 * 10, **NORM)
        T("conv", cs.conv_bwd_weight, self.d2, self.p1, self.ga2, self.gw2, self.ws)
        T("conv", cs.conv_bwd_data, self.d2, self.ga2, self.w2, self.gp1, self.ws)
        T("other", cs.net_pool_bwd, self.n1, self.gp1, self.gn1, N * K1, 28, 28)
        T("other", cs.net_norm_bwd, self.a1, self.n1, self.s1, self.gn1, self.ga1, N, K1, 28 * 28, **NORM)
        T("conv", cs.conv_bwd_weight, self.d1, x, self.ga1, self.gw1, self.ws)   # the first layer needs no input gradient
        if update:
            for w, g in ((self.w1, self.gw1), (self.w2, self.gw2), (self.wf, self.gwf), (self.bf, self.gbf)):
                T("other", cs.net_sgd_update, w, g, self.lr, w.numel())

    def times_ms(self):
        """(conv ms, other ms) of the last step; synchronises."""
        self.torch.cuda.synchronize()
        out = {"conv": 0.0, "other": 0.0}
        for kind, a, b in self.timeline:
            out[kind] += a.elapsed_time(b)
        return out["conv"], out["other"]
