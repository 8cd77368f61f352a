"""The C-ABI library loads, exports what include/*.h declare, and rejects bad
arguments before touching the GPU (none of these calls launches anything)."""
import ctypes
import os
import re

import pytest

import paper_1712_02546_amd as cs
from paper_1712_02546_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = set()
    inc = os.path.join(ROOT, "include")
    for header in sorted(os.listdir(inc)):
        if not header.endswith(".h"):
            continue
        text = open(os.path.join(inc, header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b((?:conv|net)_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    lib = cs.load()
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings():
    for code in range(-9, 1):
        assert cs.status_string(code)
    assert cs.status_string(0) == "ok"
    assert "unknown" in cs.status_string(-99)


GOOD = dict(N=8, C=3, H=32, W=32, K=16, R=5, S=5)


def test_output_dims_and_workspace_query():
    assert cs.conv_output_dims(cs.ConvDesc(**GOOD)) == (28, 28)
    assert cs.conv_output_dims(cs.ConvDesc(64, 3, 224, 224, 96, 11, 11, 4, 4, 2, 2)) == (55, 55)
    assert cs.conv_output_dims(cs.ConvDesc(1, 1, 34, 34, 1, 5, 5, 4, 4)) == (8, 8)
    for p in (cs.PASS_FWD, cs.PASS_BWD_DATA, cs.PASS_BWD_WEIGHT):
        assert cs.conv_workspace_bytes(cs.ConvDesc(**GOOD), p) > 0
        assert cs.conv_workspace_bytes(cs.ConvDesc(**GOOD, k0=3, k1=3), p) == 0
    assert cs.conv_workspace_bytes(cs.ConvDesc(**GOOD), 7) == 0


@pytest.mark.parametrize("dtype", [cs.CONV_F32, cs.CONV_BF16])
@pytest.mark.parametrize("layer", [
    dict(N=36, C=48, H=12, W=12, K=200, R=5, S=5, pad_h=1, pad_w=1),
    dict(N=128, C=500, H=14, W=14, K=1500, R=5, S=5),
    dict(N=64, C=3, H=32, W=32, K=150, R=5, S=5),
    dict(N=1024, C=50, H=14, W=14, K=500, R=5, S=5),
    dict(N=64, C=96, H=27, W=27, K=256, R=5, S=5, pad_h=2, pad_w=2),
])
def test_workspace_never_grows_when_the_slice_shrinks(layer, dtype):
    K = layer["K"]
    for p in (cs.PASS_FWD, cs.PASS_BWD_DATA, cs.PASS_BWD_WEIGHT):
        full = cs.conv_workspace_bytes(cs.ConvDesc(**layer, dtype=dtype), p)
        last = 0
        for k1 in (1, 7, 31, 32, 33, K // 3, K // 2, K - 1, K):
            need = cs.conv_workspace_bytes(cs.ConvDesc(**layer, dtype=dtype, k0=0, k1=k1), p)
            assert last <= need <= full, (p, k1, need, full)
            last = need
            shifted = cs.conv_workspace_bytes(cs.ConvDesc(**layer, dtype=dtype, k0=K - k1, k1=K), p)
            assert shifted == need, (p, k1)


@pytest.mark.parametrize("layer", [
    dict(N=64, C=128, H=56, W=56, K=300, R=3, S=3, pad_h=1, pad_w=1),
    # tile shapes and tile-sharing schemes change with the slice: 96-row and 256-row tiles, wide input-gradient tiles
    # only where their runs are long
    dict(N=128, C=500, H=14, W=14, K=1500, R=5, S=5),
    dict(N=32, C=200, H=20, W=20, K=700, R=3, S=3, pad_h=1, pad_w=1),
    dict(N=64, C=3, H=64, W=64, K=200, R=7, S=7, stride_h=2, stride_w=2, pad_h=3, pad_w=3),
], ids=lambda d: f"C{d['C']}K{d['K']}")
def test_workspace_is_monotone_over_every_slice_size(layer):
    for dtype in (cs.CONV_F32, cs.CONV_BF16):
        for p in (cs.PASS_FWD, cs.PASS_BWD_DATA, cs.PASS_BWD_WEIGHT):
            sizes = [cs.conv_workspace_bytes(cs.ConvDesc(**layer, dtype=dtype, k0=0, k1=k1), p)
                     for k1 in range(1, layer["K"] + 1)]
            assert all(a <= b for a, b in zip(sizes, sizes[1:])), (dtype, p)


class FakeBuf:
    """Stands in for a device tensor: the calls below must fail before using it."""

    def __init__(self, ptr, nbytes=1 << 20):
        self._p, self._n = ptr, nbytes

    def data_ptr(self):
        return self._p

    def numel(self):
        return self._n

    def element_size(self):
        return 1


A = FakeBuf(0x10000)
WS = FakeBuf(0x20000, 1 << 30)


@pytest.mark.parametrize("fn", [cs.conv_fwd, cs.conv_bwd_data, cs.conv_bwd_weight])
@pytest.mark.parametrize("bad,code", [
    (dict(N=0), -2), (dict(C=-1), -2), (dict(R=33, S=33), -2), (dict(H=4), -2), (dict(stride_h=0), -2),
    (dict(pad_w=-1), -2), (dict(k0=-1), -3), (dict(k1=17), -3), (dict(k0=5, k1=4), -3), (dict(dtype=2), -4),
    (dict(N=1 << 20, C=1 << 10), -2),
])
def test_bad_descriptors_are_rejected(fn, bad, code):
    d = cs.ConvDesc(**{**GOOD, **bad})
    assert fn(d, A, A, A, WS, stream=0, raw_status=True) == code


@pytest.mark.parametrize("fn", [cs.conv_fwd, cs.conv_bwd_data, cs.conv_bwd_weight])
def test_null_misaligned_and_workspace_errors(fn):
    d = cs.ConvDesc(**GOOD)
    assert fn(d, None, A, A, WS, stream=0, raw_status=True) == -1
    assert fn(d, A, None, A, WS, stream=0, raw_status=True) == -1
    assert fn(d, A, A, None, WS, stream=0, raw_status=True) == -1
    assert fn(d, FakeBuf(0x10004), A, A, WS, stream=0, raw_status=True) == -7
    assert fn(d, A, A, A, None, stream=0, raw_status=True) == -5
    assert fn(d, A, A, A, FakeBuf(0x20000, 16), stream=0, raw_status=True) == -5
    assert fn(d, A, A, A, FakeBuf(0x20010, 1 << 30), stream=0, raw_status=True) == -5
    with pytest.raises(cs.ConvError):
        fn(d, None, A, A, WS, stream=0)


def test_filter_extent_limit_is_on_the_product_only():
    """R*S <= 1024 is the documented limit: long thin filters are admitted, one tap more is not."""
    for R, S in ((1024, 1), (1, 1024), (33, 31), (64, 16)):
        d = cs.ConvDesc(N=2, C=64, H=R + 4, W=S + 4, K=4, R=R, S=S)
        assert cs.conv_output_dims(d) == (5, 5)
        for p in (cs.PASS_FWD, cs.PASS_BWD_DATA, cs.PASS_BWD_WEIGHT):
            assert cs.conv_workspace_bytes(d, p) > 0
    for R, S in ((1025, 1), (33, 32), (1, 1025)):
        d = cs.ConvDesc(N=2, C=64, H=R + 4, W=S + 4, K=4, R=R, S=S)
        assert cs.conv_fwd(d, A, A, A, WS, stream=0, raw_status=True) == -2
        assert cs.conv_bwd_data(d, A, A, A, WS, stream=0, raw_status=True) == -2


def test_noalloc_forward_rejects_before_any_launch():
    """conv_fwd_noalloc: argument errors as conv_fwd, and a layer whose workspace exceeds the
    library's fixed array is refused (none of these calls reaches the GPU)."""
    assert cs.conv_fwd_noalloc(cs.ConvDesc(**{**GOOD, "N": 0}), A, A, A, stream=0, raw_status=True) == -2
    assert cs.conv_fwd_noalloc(cs.ConvDesc(**GOOD), None, A, A, stream=0, raw_status=True) == -1
    assert cs.conv_fwd_noalloc(cs.ConvDesc(**GOOD, k0=5, k1=4), A, A, A, stream=0, raw_status=True) == -3
    big = cs.ConvDesc(N=128, C=500, H=14, W=14, K=1500, R=5, S=5)
    assert cs.conv_workspace_bytes(big, cs.PASS_FWD) > cs.NOALLOC_MAX_WORKSPACE
    assert cs.conv_fwd_noalloc(big, A, A, A, stream=0, raw_status=True) == -5
    assert cs.conv_fwd_noalloc(cs.ConvDesc(**GOOD, k0=4, k1=4), A, A, A, stream=0, raw_status=True) == 0


def test_pass_path_names_the_kernel_family():
    first = cs.ConvDesc(N=128, C=3, H=32, W=32, K=500, R=5, S=5)
    second = cs.ConvDesc(N=128, C=500, H=14, W=14, K=1500, R=5, S=5)
    assert cs.conv_pass_path(first, cs.PASS_FWD).startswith("fwd_pm_gemm_kernel: fp32 MFMA")
    assert cs.conv_pass_path(first, cs.PASS_BWD_DATA).startswith("bwd_data_pm_gemm_kernel")
    assert cs.conv_pass_path(second, cs.PASS_FWD).startswith("fwd_gemm_kernel: fp32 MFMA")
    assert cs.conv_pass_path(second, cs.PASS_BWD_DATA).startswith("bwd_data_gemm_kernel")
    bf = cs.ConvDesc(N=64, C=3, H=224, W=224, K=96, R=11, S=11, stride_h=4, stride_w=4, pad_h=2, pad_w=2, dtype=cs.CONV_BF16)
    assert cs.conv_pass_path(bf, cs.PASS_FWD).startswith("fwd16_pm_gemm_kernel: bf16 MFMA")
    assert cs.conv_pass_path(bf, cs.PASS_BWD_DATA).startswith("bwd_data16_pm_gemm_kernel: bf16 MFMA")
    assert cs.conv_pass_path(bf, cs.PASS_BWD_WEIGHT).startswith("bwd_weight16_gemm_kernel: bf16 MFMA")
    assert cs.conv_pass_path(second, 9) == "unknown pass"
    assert cs.conv_pass_path(cs.ConvDesc(N=0, C=3, H=32, W=32, K=5, R=5, S=5), 0) == "invalid descriptor"


def test_pass_path_names_the_bf16_tile_shape():
    """256 x 256 tiles for slices of more than 128 rows; the input gradient takes them only where its runs are long
    or its tiles outnumber the compute units."""
    big = dict(N=128, C=500, H=14, W=14, K=1500, R=5, S=5, dtype=cs.CONV_BF16)
    for p in (cs.PASS_FWD, cs.PASS_BWD_DATA, cs.PASS_BWD_WEIGHT):
        assert "_wide_gemm_kernel" in cs.conv_pass_path(cs.ConvDesc(**big), p), p
    share = cs.ConvDesc(**big, k0=500, k1=1000)          # a third of the kernels: short runs
    assert "_wide_gemm_kernel" in cs.conv_pass_path(share, cs.PASS_FWD)
    assert cs.conv_pass_path(share, cs.PASS_BWD_DATA).startswith("bwd_data16_gemm_kernel")
    small = cs.ConvDesc(**big, k0=0, k1=128)             # 128 kernels: one narrow row tile
    assert cs.conv_pass_path(small, cs.PASS_FWD).startswith("fwd16_gemm_kernel")
    assert cs.conv_pass_path(small, cs.PASS_BWD_WEIGHT).startswith("bwd_weight16_gemm_kernel")
    c96 = cs.ConvDesc(N=64, C=96, H=27, W=27, K=256, R=5, S=5, pad_h=2, pad_w=2, dtype=cs.CONV_BF16)
    assert "_wide_gemm_kernel" in cs.conv_pass_path(c96, cs.PASS_FWD)
    assert cs.conv_pass_path(c96, cs.PASS_BWD_DATA).startswith("bwd_data16_gemm_kernel")   # 96 channels: narrow rows


def test_null_descriptor():
    lib = cs.load()
    assert lib.conv_fwd(None, 1, 1, 1, 1, 0, None) == -1
    assert lib.conv_workspace_bytes(None, 0) == 0
    p = ctypes.c_int32()
    assert lib.conv_output_dims(None, ctypes.byref(p), ctypes.byref(p)) == -1


def test_empty_slice_needs_no_workspace_for_fwd_and_bwd_weight():
    d = cs.ConvDesc(**GOOD, k0=4, k1=4)
    assert cs.conv_fwd(d, A, A, A, None, stream=0, raw_status=True) == 0
    assert cs.conv_bwd_weight(d, A, A, A, None, stream=0, raw_status=True) == 0
    da = cs.ConvDesc(**GOOD, k0=4, k1=4, accumulate=1)
    assert cs.conv_bwd_data(da, A, A, A, None, stream=0, raw_status=True) == 0


def test_loading_the_library_brings_in_torch_first():
    """PyTorch-ROCm ships its own HIP runtime; the binding must not let the system copy in
    ahead of it (two runtimes in one process crash at the first kernel launch)."""
    import subprocess
    import sys
    code = ("import sys; import paper_1712_02546_amd as cs; assert 'torch' not in sys.modules; "
            "cs.load(); assert 'torch' in sys.modules; "
            "maps = open('/proc/self/maps').read(); "
            "libs = {l.split()[-1] for l in maps.splitlines() if 'libamdhip64' in l}; "
            "assert len(libs) == 1, libs")
    subprocess.check_call([sys.executable, "-c", code], cwd=ROOT)


def test_net_layer_calls_reject_bad_arguments():
    B = FakeBuf(0x30000)
    assert cs.net_norm_fwd(B, B, B, 2, 4, 9, size=4, stream=0, raw_status=True) == -2        # even window
    assert cs.net_norm_fwd(None, B, B, 2, 4, 9, stream=0, raw_status=True) == -1
    assert cs.net_norm_bwd(B, B, B, B, B, 0, 4, 9, stream=0, raw_status=True) == -2
    assert cs.net_pool_fwd(B, B, 6, 4, 4, win=5, stride=2, stream=0, raw_status=True) == -2   # window larger than the map
    assert cs.net_pool_bwd(B, B, None, 6, 4, 4, stream=0, raw_status=True) == -1
    assert cs.net_fc_fwd(B, B, None, B, 0, 5, 3, stream=0, raw_status=True) == -2
    assert cs.net_fc_bwd(B, None, B, B, None, None, 2, 5, 3, stream=0, raw_status=True) == -1  # dx wanted but no W
    assert cs.net_softmax_loss_fwd(B, B, None, 4, 10, stream=0, raw_status=True) == -1
    assert cs.net_softmax_loss_bwd(B, B, B, 4, 0, stream=0, raw_status=True) == -2
    assert cs.net_sgd_update(B, B, 0.1, -1, stream=0, raw_status=True) == -2
    assert cs.net_sgd_update(B, B, 0.1, 0, stream=0, raw_status=True) == 0
