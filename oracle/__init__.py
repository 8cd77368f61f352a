"""CPU oracle for the per-device convolution of arXiv 1712.02546 -- TEST INFRASTRUCTURE.

A ctypes front end to ``conv_oracle.c`` (plain direct loops, all fp64).  It is
independent of the HIP path: no shared code, headers or helpers, and it must
only be used by ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline``
leg of ``bench.py``.

Functions follow Section 4.1.2 / Algorithms 1-2 (one device convolves all input
maps with its own block ``[k0,k1)`` of the layer's kernels) and the abstract
(backward convolutions are part of the distributed work).  ``y``, ``dy``, ``w``
and ``dw`` are full-layer arrays; only channels of the slice are produced, the
rest is returned as zeros.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv_oracle.c")
_LIB = os.path.join(_HERE, "libconv_oracle.so")


def build(force: bool = False) -> str:
    """Compile conv_oracle.c with gcc (host only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11", "-Wall", "-Wextra",
             "-o", _LIB, _SRC])
    return _LIB


def use_native_build() -> str:
    """For the timed baseline only: the same source compiled ``-O3 -march=native`` for the
    host this process runs on, into a temporary directory, and used from then on in this
    process.  Returns the compiler flags used.  (The in-tree build stays portable, because
    it is built on one machine and may be loaded on another.)"""
    global _lib
    import tempfile
    flags = ["-O3", "-march=native", "-fopenmp"]
    out = os.path.join(tempfile.mkdtemp(prefix="conv_oracle_"), "libconv_oracle_native.so")
    subprocess.check_call(["gcc"] + flags + ["-shared", "-fPIC", "-std=c11", "-o", out, _SRC])
    _lib = None
    _load(out)
    return " ".join(flags)


class _Shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("N", "C", "H", "W", "K", "R", "S", "sh", "sw", "ph", "pw", "k0", "k1")]


@dataclass(frozen=True)
class Shape:
    N: int
    C: int
    H: int
    W: int
    K: int
    R: int
    S: int
    sh: int = 1
    sw: int = 1
    ph: int = 0
    pw: int = 0
    k0: int = 0
    k1: int = -1  # -1: whole layer

    def resolved(self) -> "Shape":
        if self.k1 >= 0:
            return self
        return Shape(self.N, self.C, self.H, self.W, self.K, self.R, self.S,
                     self.sh, self.sw, self.ph, self.pw, self.k0, self.K)

    def _c(self) -> _Shape:
        s = self.resolved()
        return _Shape(s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.sh, s.sw, s.ph, s.pw, s.k0, s.k1)


_lib = None


def _load(path: str | None = None):
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(path or build())
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int64)
        sp = ctypes.POINTER(_Shape)
        for name in ("oracle_conv_fwd", "oracle_conv_bwd_data", "oracle_conv_bwd_weight"):
            f = getattr(lib, name)
            f.argtypes = [sp, dp, dp, dp]
            f.restype = ctypes.c_int
        for name in ("oracle_conv_fwd_at", "oracle_conv_bwd_data_at", "oracle_conv_bwd_weight_at"):
            f = getattr(lib, name)
            f.argtypes = [sp, dp, dp, ip, ctypes.c_int64, dp]
            f.restype = ctypes.c_int
        lib.oracle_out_hw.argtypes = [sp, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32)]
        lib.oracle_out_hw.restype = ctypes.c_int
        lib.oracle_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def threads() -> int:
    """OpenMP threads the loops will use."""
    return int(_load().oracle_threads())


def out_hw(sh: Shape) -> tuple[int, int]:
    p, q = ctypes.c_int32(), ctypes.c_int32()
    cs = sh._c()
    if _load().oracle_out_hw(ctypes.byref(cs), ctypes.byref(p), ctypes.byref(q)) != 0:
        raise ValueError(f"invalid shape {sh}")
    return int(p.value), int(q.value)


def _f64(a, shape) -> np.ndarray:
    a = np.ascontiguousarray(np.asarray(a), dtype=np.float64)  # float32 -> float64 is exact
    if a.shape != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {a.shape}")
    return a


def _dp(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def conv_fwd(sh: Shape, x, w) -> np.ndarray:
    """y[N,K,P,Q] in fp64; channels outside [k0,k1) are zero."""
    sh = sh.resolved()
    P, Q = out_hw(sh)
    x = _f64(x, (sh.N, sh.C, sh.H, sh.W))
    w = _f64(w, (sh.K, sh.C, sh.R, sh.S))
    y = np.zeros((sh.N, sh.K, P, Q), dtype=np.float64)
    cs = sh._c()
    if _load().oracle_conv_fwd(ctypes.byref(cs), _dp(x), _dp(w), _dp(y)) != 0:
        raise ValueError("oracle_conv_fwd rejected its arguments")
    return y


def conv_bwd_data(sh: Shape, dy, w) -> np.ndarray:
    """dx[N,C,H,W] in fp64: the sum over the kernels of the slice only."""
    sh = sh.resolved()
    P, Q = out_hw(sh)
    dy = _f64(dy, (sh.N, sh.K, P, Q))
    w = _f64(w, (sh.K, sh.C, sh.R, sh.S))
    dx = np.zeros((sh.N, sh.C, sh.H, sh.W), dtype=np.float64)
    cs = sh._c()
    if _load().oracle_conv_bwd_data(ctypes.byref(cs), _dp(dy), _dp(w), _dp(dx)) != 0:
        raise ValueError("oracle_conv_bwd_data rejected its arguments")
    return dx


def conv_bwd_weight(sh: Shape, x, dy) -> np.ndarray:
    """dw[K,C,R,S] in fp64; rows outside [k0,k1) are zero."""
    sh = sh.resolved()
    P, Q = out_hw(sh)
    x = _f64(x, (sh.N, sh.C, sh.H, sh.W))
    dy = _f64(dy, (sh.N, sh.K, P, Q))
    dw = np.zeros((sh.K, sh.C, sh.R, sh.S), dtype=np.float64)
    cs = sh._c()
    if _load().oracle_conv_bwd_weight(ctypes.byref(cs), _dp(x), _dp(dy), _dp(dw)) != 0:
        raise ValueError("oracle_conv_bwd_weight rejected its arguments")
    return dw


def _at(fn_name: str, sh: Shape, a, a_shape, b, b_shape, idx) -> np.ndarray:
    a = _f64(a, a_shape)
    b = _f64(b, b_shape)
    idx = np.ascontiguousarray(np.asarray(idx).reshape(-1), dtype=np.int64)
    out = np.zeros(idx.shape[0], dtype=np.float64)
    cs = sh._c()
    rc = getattr(_load(), fn_name)(
        ctypes.byref(cs), _dp(a), _dp(b),
        idx.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), idx.shape[0], _dp(out))
    if rc != 0:
        raise ValueError(f"{fn_name} rejected its arguments (rc={rc})")
    return out


def conv_fwd_at(sh: Shape, x, w, idx) -> np.ndarray:
    """Elements of y at flat indices ``idx`` (row-major over [N,K,P,Q])."""
    sh = sh.resolved()
    return _at("oracle_conv_fwd_at", sh, x, (sh.N, sh.C, sh.H, sh.W),
               w, (sh.K, sh.C, sh.R, sh.S), idx)


def conv_bwd_data_at(sh: Shape, dy, w, idx) -> np.ndarray:
    """Elements of dx at flat indices ``idx`` (row-major over [N,C,H,W])."""
    sh = sh.resolved()
    P, Q = out_hw(sh)
    return _at("oracle_conv_bwd_data_at", sh, dy, (sh.N, sh.K, P, Q),
               w, (sh.K, sh.C, sh.R, sh.S), idx)


def conv_bwd_weight_at(sh: Shape, x, dy, idx) -> np.ndarray:
    """Elements of dw at flat indices ``idx`` (row-major over [K,C,R,S])."""
    sh = sh.resolved()
    P, Q = out_hw(sh)
    return _at("oracle_conv_bwd_weight_at", sh, x, (sh.N, sh.C, sh.H, sh.W),
               dy, (sh.N, sh.K, P, Q), idx)
