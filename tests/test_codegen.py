"""Properties of the generated gfx950 code that the performance of the matrix-core kernels
rests on and that a source change can silently lose: no register spills to scratch memory,
and few enough registers for two workgroups per compute unit."""
import os
import re
import subprocess

import pytest

from paper_1712_02546_amd import build as cbuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def device_asm(tmp_path_factory):
    out = tmp_path_factory.mktemp("asm") / "convslice.s"
    flags = [f for f in cbuild.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")] + flags + ["-S", "--cuda-device-only", "-o", str(out),
                                                                      cbuild.SOURCES[0]]
    subprocess.check_call(cmd, stderr=subprocess.DEVNULL)
    return out.read_text()


def kernel_stats(asm):
    """name -> {ScratchSize, TotalNumVgprs, ...} from the per-kernel comment block the compiler emits."""
    stats = {}
    blocks = re.split(r"^\s*\.amdhsa_kernel\s+", asm, flags=re.M)
    for blk in blocks[1:]:
        name = blk.split()[0]
        tail = blk.split(".end_amdhsa_kernel", 1)[1] if ".end_amdhsa_kernel" in blk else ""
        d = {k: int(v) for k, v in re.findall(r";\s*(ScratchSize|TotalNumVgprs|NumVgprs|NumAgprs|Occupancy):\s*(\d+)", tail)}
        stats[name] = d
    return stats


def test_matrix_core_kernels_do_not_spill_and_fit_two_workgroups_per_cu(device_asm):
    stats = kernel_stats(device_asm)
    gemm = {n: s for n, s in stats.items() if "gemm_kernel" in n}
    assert len(gemm) >= 8, sorted(stats)        # fwd x2, bwd_data, bwd_weight x2, three bf16 kernels
    for name, s in gemm.items():
        assert s.get("ScratchSize") == 0, (name, s)
        assert s.get("TotalNumVgprs", 999) <= 256, (name, s)   # 512 registers per SIMD lane, two waves per SIMD


def test_operand_staging_uses_lds_dma_with_scalar_bases(device_asm):
    # the 16-byte global->LDS load, in the form that takes its base from scalar registers
    assert len(re.findall(r"global_load_lds_dwordx4 v\d+, s\[\d+:\d+\]", device_asm)) >= 40
