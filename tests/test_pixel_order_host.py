"""The input-gradient set-up logic (csrc/pixel_order.h) built for the host with
-fsanitize=address,undefined and run on bounds-checked tables of exactly the extents the GPU
kernel declares: for filter extents up to the library's limit (R*S <= 1024, so R or S up to
1024), strides 1-4 and pads 0-3, no table access is out of bounds, perm is a permutation with
non-increasing tap counts, and pre is the running sum of the tile lengths."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def host_check(tmp_path_factory):
    exe = tmp_path_factory.mktemp("po") / "pixel_order_host"
    subprocess.check_call(["g++", "-std=c++17", "-O2", "-g", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", "-o", str(exe),
                           os.path.join(ROOT, "tests", "pixel_order_host.cpp")])
    return str(exe)


@pytest.mark.parametrize("mode", [0, 1], ids=["sweep", "limits"])
def test_pixel_order_tables_stay_in_bounds_and_order_is_valid(host_check, mode):
    r = subprocess.run([host_check, str(mode)], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.startswith("ok "), r.stdout


@pytest.mark.parametrize("geom", [
    # H  W   R   S  sh sw ph pw NB nkc T   -- shapes that overran fixed 34/1056-entry tables
    (40, 10, 33, 3, 1, 1, 0, 0, 1, 1, 1024),
    (70, 4, 64, 1, 1, 1, 0, 0, 1, 2, 1024),
    (1030, 3, 1024, 1, 1, 1, 0, 0, 1, 1, 1024),
    (34, 34, 32, 32, 1, 1, 0, 0, 1, 1, 1024),
])
def test_long_filters_on_the_per_pixel_path(host_check, geom):
    r = subprocess.run([host_check] + [str(v) for v in geom], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout + r.stderr
