"""ctypes binding of libconvslice.so: same names as the C ABI, argument marshalling only.

Tensors are PyTorch-ROCm tensors used as plain device buffers (``data_ptr()``);
the stream is torch's current HIP stream unless one is given.  There is no
fallback: if the library has not been built, importing the symbols raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("CONVSLICE_LIB") or os.path.join(_HERE, "libconvslice.so")

CONV_F32, CONV_BF16 = 0, 1
PASS_FWD, PASS_BWD_DATA, PASS_BWD_WEIGHT = 0, 1, 2

NOALLOC_MAX_WORKSPACE = 96 << 20

EXPORTS = ("conv_output_dims", "conv_workspace_bytes", "conv_fwd", "conv_fwd_noalloc", "conv_bwd_data",
           "conv_bwd_weight", "conv_status_string", "conv_probe_next_call", "conv_pass_path",
           "conv_partition", "conv_partition_estimate", "conv_calibrate_workspace_bytes",
           "conv_calibrate", "conv_layer_workspace_bytes", "conv_layer_fwd",
           "conv_layer_bwd_data", "conv_layer_bwd_weight", "conv_comm_elements",
           "conv_comm_elements_partition", "conv_scaling_estimate",
           "net_norm_fwd", "net_norm_bwd", "net_pool_fwd", "net_pool_bwd", "net_fc_fwd", "net_fc_bwd",
           "net_softmax_loss_fwd", "net_softmax_loss_bwd", "net_sgd_update")
MAX_DEVICES = 64


class conv_desc_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "N", "C", "H", "W", "K", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w",
        "k0", "k1", "dtype", "accumulate")]


class conv_comm_layer_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("inp", "inCh", "k", "numK", "out")]


@dataclass(frozen=True)
class ConvDesc:
    """Host-side mirror of conv_desc_t (k1 = -1 means the whole layer)."""
    N: int
    C: int
    H: int
    W: int
    K: int
    R: int
    S: int
    stride_h: int = 1
    stride_w: int = 1
    pad_h: int = 0
    pad_w: int = 0
    k0: int = 0
    k1: int = -1
    dtype: int = CONV_F32
    accumulate: int = 0

    def c_struct(self) -> conv_desc_t:
        k1 = self.K if self.k1 < 0 else self.k1
        return conv_desc_t(self.N, self.C, self.H, self.W, self.K, self.R, self.S,
                           self.stride_h, self.stride_w, self.pad_h, self.pad_w,
                           self.k0, k1, self.dtype, self.accumulate)


class ConvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({status_string(status)})")


_lib = None


def load() -> ctypes.CDLL:
    """Load libconvslice.so; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_1712_02546_amd.build` "
                "(hipcc, gfx950). There is no CPU or PyTorch fallback.")
        # PyTorch-ROCm carries its own copy of the HIP runtime.  If this library were loaded
        # first it would pull in the system copy, a later `import torch` would add a second
        # one, and the first kernel launch would crash inside the duplicated runtime.
        import torch  # noqa: F401
        lib = ctypes.CDLL(LIB_PATH)
        dp = ctypes.POINTER(conv_desc_t)
        vp = ctypes.c_void_p
        lib.conv_output_dims.argtypes = [dp, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32)]
        lib.conv_output_dims.restype = ctypes.c_int
        lib.conv_workspace_bytes.argtypes = [dp, ctypes.c_int]
        lib.conv_workspace_bytes.restype = ctypes.c_size_t
        for name in ("conv_fwd", "conv_bwd_data", "conv_bwd_weight"):
            f = getattr(lib, name)
            f.argtypes = [dp, vp, vp, vp, vp, ctypes.c_size_t, vp]
            f.restype = ctypes.c_int
        lib.conv_fwd_noalloc.argtypes = [dp, vp, vp, vp, vp]
        lib.conv_fwd_noalloc.restype = ctypes.c_int
        lib.conv_probe_next_call.argtypes = [vp, vp]
        lib.conv_probe_next_call.restype = ctypes.c_int
        lib.conv_pass_path.argtypes = [dp, ctypes.c_int]
        lib.conv_pass_path.restype = ctypes.c_char_p
        lib.conv_status_string.argtypes = [ctypes.c_int]
        lib.conv_status_string.restype = ctypes.c_char_p
        pd, pi = ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int32)
        lib.conv_partition.argtypes = [pd, ctypes.c_int32, ctypes.c_int32, pd, pi]
        lib.conv_partition.restype = ctypes.c_int
        lib.conv_partition_estimate.argtypes = [pd, pd, ctypes.c_int32, pd, pd]
        lib.conv_partition_estimate.restype = ctypes.c_int
        lib.conv_calibrate_workspace_bytes.argtypes = [dp, ctypes.c_int]
        lib.conv_calibrate_workspace_bytes.restype = ctypes.c_size_t
        lib.conv_calibrate.argtypes = [dp, ctypes.c_int, ctypes.c_int, vp, ctypes.c_size_t, vp, pd]
        lib.conv_calibrate.restype = ctypes.c_int
        lib.conv_layer_workspace_bytes.argtypes = [dp, pi, ctypes.c_int32, ctypes.c_int]
        lib.conv_layer_workspace_bytes.restype = ctypes.c_size_t
        pl = ctypes.POINTER(conv_comm_layer_t)
        lib.conv_comm_elements.argtypes = [pl, ctypes.c_int32, ctypes.c_int64, pd]
        lib.conv_comm_elements.restype = ctypes.c_int
        lib.conv_comm_elements_partition.argtypes = [pl, ctypes.c_int64, pi, ctypes.c_int32, ctypes.c_int32, pd]
        lib.conv_comm_elements_partition.restype = ctypes.c_int
        lib.conv_scaling_estimate.argtypes = [pd, pd, ctypes.c_int32, ctypes.c_int32] + [ctypes.c_double] * 4 + [pd] * 3
        lib.conv_scaling_estimate.restype = ctypes.c_int
        i32, f32 = ctypes.c_int32, ctypes.c_float
        lib.net_norm_fwd.argtypes = [vp, vp, vp, i32, i32, i32, i32, f32, f32, f32, vp]
        lib.net_norm_bwd.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, f32, f32, f32, vp]
        lib.net_pool_fwd.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp]
        lib.net_pool_bwd.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, vp]
        lib.net_fc_fwd.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp]
        lib.net_fc_bwd.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, vp]
        lib.net_softmax_loss_fwd.argtypes = [vp, vp, vp, i32, i32, vp]
        lib.net_softmax_loss_bwd.argtypes = [vp, vp, vp, i32, i32, vp]
        lib.net_sgd_update.argtypes = [vp, vp, f32, ctypes.c_int64, vp]
        for name in EXPORTS:
            if name.startswith("net_"):
                getattr(lib, name).restype = ctypes.c_int
        for name in ("conv_layer_fwd", "conv_layer_bwd_data", "conv_layer_bwd_weight"):
            f = getattr(lib, name)
            f.argtypes = [dp, pi, ctypes.c_int32, vp, vp, vp, vp, ctypes.c_size_t, vp]
            f.restype = ctypes.c_int
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load().conv_status_string(int(status)).decode()


def conv_pass_path(desc: "ConvDesc", which: int) -> str:
    """Kernel family that serves the pass: "<matrix-core kernel>: <arithmetic>, <layout>"."""
    cd = desc.c_struct()
    return load().conv_pass_path(ctypes.byref(cd), int(which)).decode()


def conv_probe_next_call(start_event, stop_event) -> int:
    """Arm the one-shot matrix-core-kernel timing probe with two raw hipEvent_t handles (ints)."""
    return int(load().conv_probe_next_call(start_event, stop_event))


def conv_output_dims(desc: ConvDesc) -> tuple[int, int]:
    p, q = ctypes.c_int32(), ctypes.c_int32()
    cd = desc.c_struct()
    rc = load().conv_output_dims(ctypes.byref(cd), ctypes.byref(p), ctypes.byref(q))
    if rc != 0:
        raise ConvError(rc, "conv_output_dims")
    return int(p.value), int(q.value)


def conv_workspace_bytes(desc: ConvDesc, which: int) -> int:
    cd = desc.c_struct()
    return int(load().conv_workspace_bytes(ctypes.byref(cd), int(which)))


def _ptr(t) -> int:
    return 0 if t is None else int(t.data_ptr())


def _stream(stream) -> int:
    if stream is not None:
        return int(stream)
    import torch
    return int(torch.cuda.current_stream().cuda_stream)


def _call(name: str, desc: ConvDesc, a, b, out, ws, stream, raw_status: bool):
    cd = desc.c_struct()
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    rc = getattr(load(), name)(ctypes.byref(cd), _ptr(a), _ptr(b), _ptr(out), _ptr(ws), ws_bytes,
                               _stream(stream))
    if raw_status:
        return rc
    if rc != 0:
        raise ConvError(rc, name)
    return out


def conv_fwd(desc: ConvDesc, x, w, y, ws=None, stream=None, raw_status=False):
    """y[:, k0:k1] = conv(x, w[k0:k1]) enqueued on the stream; returns y."""
    return _call("conv_fwd", desc, x, w, y, ws, stream, raw_status)


def conv_fwd_noalloc(desc: ConvDesc, x, w, y, stream=None, raw_status=False):
    """conv_fwd on the library's own fixed scratch array (layers up to NOALLOC_MAX_WORKSPACE); returns y."""
    cd = desc.c_struct()
    rc = load().conv_fwd_noalloc(ctypes.byref(cd), _ptr(x), _ptr(w), _ptr(y), _stream(stream))
    if raw_status:
        return rc
    if rc != 0:
        raise ConvError(rc, "conv_fwd_noalloc")
    return y


def conv_bwd_data(desc: ConvDesc, dy, w, dx, ws=None, stream=None, raw_status=False):
    """dx (+)= input gradient from dy[:, k0:k1] and w[k0:k1]; returns dx."""
    return _call("conv_bwd_data", desc, dy, w, dx, ws, stream, raw_status)


def conv_bwd_weight(desc: ConvDesc, x, dy, dw, ws=None, stream=None, raw_status=False):
    """dw[k0:k1] = weight gradient from x and dy[:, k0:k1]; returns dw (fp32)."""
    return _call("conv_bwd_weight", desc, x, dy, dw, ws, stream, raw_status)


# ---- convlayer.h: Eq. (1) partition, calibration probe, partitioned layer --------------------

def _doubles(v):
    return (ctypes.c_double * len(v))(*[float(a) for a in v])


def _ints(v):
    return (ctypes.c_int32 * len(v))(*[int(a) for a in v])


def conv_partition(t, K: int, raw_status=False):
    """Eq. (1) shares and contiguous k-bounds for probe times t; returns (shares, bounds)."""
    n = len(t)
    shares = (ctypes.c_double * max(n, 1))()
    bounds = (ctypes.c_int32 * (max(n, 0) + 1))()
    rc = load().conv_partition(_doubles(t) if n else None, n, int(K), shares, bounds)
    if raw_status:
        return rc
    if rc != 0:
        raise ConvError(rc, "conv_partition")
    return [float(v) for v in shares[:n]], [int(v) for v in bounds[:n + 1]]


def conv_partition_estimate(t, shares, raw_status=False):
    """(finish time of the slowest device, speed-up over the fastest device alone)."""
    fin, sp = ctypes.c_double(), ctypes.c_double()
    rc = load().conv_partition_estimate(_doubles(t), _doubles(shares), len(t), ctypes.byref(fin),
                                        ctypes.byref(sp))
    if raw_status:
        return rc
    if rc != 0:
        raise ConvError(rc, "conv_partition_estimate")
    return float(fin.value), float(sp.value)


def pass_mask(*passes: int) -> int:
    m = 0
    for p in passes:
        m |= 1 << p
    return m


def conv_calibrate_workspace_bytes(desc: ConvDesc, mask: int) -> int:
    cd = desc.c_struct()
    return int(load().conv_calibrate_workspace_bytes(ctypes.byref(cd), int(mask)))


def conv_calibrate(desc: ConvDesc, mask: int, reps: int, ws, stream=None, raw_status=False):
    """Seconds per repetition of the selected passes on random data (blocks until measured)."""
    cd = desc.c_struct()
    sec = ctypes.c_double()
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    rc = load().conv_calibrate(ctypes.byref(cd), int(mask), int(reps), _ptr(ws), ws_bytes,
                               _stream(stream), ctypes.byref(sec))
    if raw_status:
        return rc
    if rc != 0:
        raise ConvError(rc, "conv_calibrate")
    return float(sec.value)


def conv_layer_workspace_bytes(desc: ConvDesc, bounds, which: int) -> int:
    cd = desc.c_struct()
    return int(load().conv_layer_workspace_bytes(ctypes.byref(cd), _ints(bounds), len(bounds) - 1, int(which)))


def _layer_call(name: str, desc: ConvDesc, bounds, a, b, out, ws, stream, raw_status: bool):
    cd = desc.c_struct()
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    rc = getattr(load(), name)(ctypes.byref(cd), _ints(bounds), len(bounds) - 1, _ptr(a), _ptr(b), _ptr(out),
                               _ptr(ws), ws_bytes, _stream(stream))
    if raw_status:
        return rc
    if rc != 0:
        raise ConvError(rc, name)
    return out


def conv_layer_fwd(desc: ConvDesc, bounds, x, w, y, ws=None, stream=None, raw_status=False):
    """All slices of the partition `bounds` write their channel blocks of y; returns y."""
    return _layer_call("conv_layer_fwd", desc, bounds, x, w, y, ws, stream, raw_status)


def conv_layer_bwd_data(desc: ConvDesc, bounds, dy, w, dx, ws=None, stream=None, raw_status=False):
    """dx (+)= sum of the slices' partial input gradients, in slice order; returns dx."""
    return _layer_call("conv_layer_bwd_data", desc, bounds, dy, w, dx, ws, stream, raw_status)


def conv_layer_bwd_weight(desc: ConvDesc, bounds, x, dy, dw, ws=None, stream=None, raw_status=False):
    """All slices of the partition write their blocks of dw; returns dw (fp32)."""
    return _layer_call("conv_layer_bwd_weight", desc, bounds, x, dy, dw, ws, stream, raw_status)


# ---- convlayer.h: Eq. (2) communication volume and the scalability estimate -------------------

def conv_comm_elements(layers, batch: int, raw_status=False):
    """Eq. (2): elements exchanged per batch; layers are (in, inCh, k, numK, out) tuples."""
    arr = (conv_comm_layer_t * max(len(layers), 1))(*[conv_comm_layer_t(*l) for l in layers])
    out = ctypes.c_double()
    rc = load().conv_comm_elements(arr, len(layers), int(batch), ctypes.byref(out))
    if raw_status:
        return rc
    if rc != 0:
        raise ConvError(rc, "conv_comm_elements")
    return float(out.value)


def conv_comm_elements_partition(layer, batch: int, bounds, master: int = 0, raw_status=False):
    """Elements the master exchanges for one layer split at `bounds` (its own block stays home)."""
    l = conv_comm_layer_t(*layer)
    out = ctypes.c_double()
    rc = load().conv_comm_elements_partition(ctypes.byref(l), int(batch), _ints(bounds), len(bounds) - 1,
                                             int(master), ctypes.byref(out))
    if raw_status:
        return rc
    if rc != 0:
        raise ConvError(rc, "conv_comm_elements_partition")
    return float(out.value)


def conv_scaling_estimate(t_conv, shares, t_comp: float, elements: float, bytes_per_element: float,
                          bits_per_second: float, master: int = 0, raw_status=False):
    """(seconds per batch, speed-up over the master alone, Amdahl bound) of Section 4.2's model."""
    sec, sp, am = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
    rc = load().conv_scaling_estimate(_doubles(t_conv), _doubles(shares), len(t_conv), int(master), float(t_comp),
                                      float(elements), float(bytes_per_element), float(bits_per_second),
                                      ctypes.byref(sec), ctypes.byref(sp), ctypes.byref(am))
    if raw_status:
        return rc
    if rc != 0:
        raise ConvError(rc, "conv_scaling_estimate")
    return float(sec.value), float(sp.value), float(am.value)


# ---- convnet.h: the network's other layers (fp32 device tensors) ------------------------------

def _net(name, raw_status, *args):
    rc = getattr(load(), name)(*args)
    if raw_status:
        return rc
    if rc != 0:
        raise ConvError(rc, name)
    return None


def net_norm_fwd(x, y, scale, N, C, HW, size=5, kappa=1.0, alpha=1e-4, beta=0.75, stream=None, raw_status=False):
    return _net("net_norm_fwd", raw_status, _ptr(x), _ptr(y), _ptr(scale), N, C, HW, size, kappa, alpha, beta,
                _stream(stream))


def net_norm_bwd(x, y, scale, dy, dx, N, C, HW, size=5, kappa=1.0, alpha=1e-4, beta=0.75, stream=None,
                 raw_status=False):
    return _net("net_norm_bwd", raw_status, _ptr(x), _ptr(y), _ptr(scale), _ptr(dy), _ptr(dx), N, C, HW, size, kappa,
                alpha, beta, _stream(stream))


def net_pool_fwd(x, y, NC, H, W, win=2, stride=2, stream=None, raw_status=False):
    return _net("net_pool_fwd", raw_status, _ptr(x), _ptr(y), NC, H, W, win, stride, _stream(stream))


def net_pool_bwd(x, dy, dx, NC, H, W, win=2, stride=2, stream=None, raw_status=False):
    return _net("net_pool_bwd", raw_status, _ptr(x), _ptr(dy), _ptr(dx), NC, H, W, win, stride, _stream(stream))


def net_fc_fwd(x, W, b, y, N, I, O, stream=None, raw_status=False):
    return _net("net_fc_fwd", raw_status, _ptr(x), _ptr(W), _ptr(b), _ptr(y), N, I, O, _stream(stream))


def net_fc_bwd(x, W, dy, dx, dW, db, N, I, O, stream=None, raw_status=False):
    return _net("net_fc_bwd", raw_status, _ptr(x), _ptr(W), _ptr(dy), _ptr(dx), _ptr(dW), _ptr(db), N, I, O,
                _stream(stream))


def net_softmax_loss_fwd(z, labels, loss, N, O, stream=None, raw_status=False):
    return _net("net_softmax_loss_fwd", raw_status, _ptr(z), _ptr(labels), _ptr(loss), N, O, _stream(stream))


def net_softmax_loss_bwd(z, labels, dz, N, O, stream=None, raw_status=False):
    return _net("net_softmax_loss_bwd", raw_status, _ptr(z), _ptr(labels), _ptr(dz), N, O, _stream(stream))


def net_sgd_update(w, dw, lr, count, stream=None, raw_status=False):
    return _net("net_sgd_update", raw_status, _ptr(w), _ptr(dw), lr, count, _stream(stream))
