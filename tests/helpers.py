"""Shared helpers for the parity tests: run the HIP path on numpy inputs, error metric."""
from __future__ import annotations

import numpy as np

import oracle
import paper_1712_02546_amd as cs
from paper_1712_02546_amd import synth

FP32_TOL = 1e-4   # max relative error, fp32 path (spec tolerance)
BF16_TOL = 2e-2   # max relative error, bf16 inputs/outputs with fp32 accumulate


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max_i |g_i - o_i| / max(|o_i|, rms(o)): element-wise relative error with the
    root-mean-square of the reference as floor, so that elements which are small only
    through cancellation are judged against the scale of the tensor."""
    got = np.asarray(got, dtype=np.float64).ravel()
    ref = np.asarray(ref, dtype=np.float64).ravel()
    if ref.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(ref * ref)))
    denom = np.maximum(np.abs(ref), rms)
    if rms == 0.0:
        return float(np.max(np.abs(got - ref)))
    return float(np.max(np.abs(got - ref) / denom))


def oracle_shape(cfg: synth.LayerConfig) -> oracle.Shape:
    k0, k1 = cfg.slice
    return oracle.Shape(cfg.N, cfg.C, cfg.H, cfg.W, cfg.K, cfg.R, cfg.S, cfg.stride, cfg.stride,
                        cfg.pad, cfg.pad, k0, k1)


def desc_of(cfg: synth.LayerConfig, dtype=cs.CONV_F32, accumulate=0) -> cs.ConvDesc:
    k0, k1 = cfg.slice
    return cs.ConvDesc(cfg.N, cfg.C, cfg.H, cfg.W, cfg.K, cfg.R, cfg.S, cfg.stride, cfg.stride,
                       cfg.pad, cfg.pad, k0, k1, dtype, accumulate)


class Device:
    """Device buffers for one configuration; torch is used for memory only."""

    def __init__(self, cfg: synth.LayerConfig, x, w, dy, dtype=cs.CONV_F32):
        import torch
        self.torch = torch
        self.cfg, self.dtype = cfg, dtype
        self.dev = torch.device("cuda:0")
        self.x = self._up(x)
        self.w = self._up(w)
        self.dy = self._up(dy)
        need = max(cs.conv_workspace_bytes(desc_of(cfg, dtype), p) for p in (0, 1, 2))
        self.ws = torch.empty(max(need, 256), dtype=torch.uint8, device=self.dev)
        assert self.ws.data_ptr() % 256 == 0

    def _up(self, a):
        torch = self.torch
        if a is None:
            return None
        if self.dtype == cs.CONV_BF16:
            bits = synth.f32_to_bf16_bits(a).view(np.int16)
            return torch.from_numpy(bits).to(self.dev).view(torch.bfloat16)
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(self.dev)

    def _empty(self, shape, fp32=False, fill=None):
        torch = self.torch
        dt = torch.float32 if (fp32 or self.dtype == cs.CONV_F32) else torch.bfloat16
        if fill is None:
            return torch.empty(shape, dtype=dt, device=self.dev)
        return torch.full(shape, fill, dtype=dt, device=self.dev)

    def _down(self, t):
        self.torch.cuda.synchronize()
        return t.float().cpu().numpy()

    def fwd(self, fill=None):
        c = self.cfg
        y = self._empty((c.N, c.K, c.P, c.Q), fill=fill)
        cs.conv_fwd(desc_of(c, self.dtype), self.x, self.w, y, self.ws)
        return self._down(y)

    def bwd_data(self, accumulate=0, init=None):
        c = self.cfg
        dx = self._empty((c.N, c.C, c.H, c.W)) if init is None else self._up(init)
        cs.conv_bwd_data(desc_of(c, self.dtype, accumulate), self.dy, self.w, dx, self.ws)
        return self._down(dx)

    def bwd_weight(self, fill=None):
        c = self.cfg
        dw = self._empty((c.K, c.C, c.R, c.S), fp32=True, fill=fill)
        cs.conv_bwd_weight(desc_of(c, self.dtype), self.x, self.dy, dw, self.ws)
        return self._down(dw)


def sample_indices(total: int, count: int, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    if total <= count:
        return np.arange(total, dtype=np.int64)
    return np.unique(rng.integers(0, total, size=count, dtype=np.int64))
