"""The C oracle built with -fsanitize=address,undefined and driven over a sweep of shapes
(strides, paddings, rectangular filters, interior and empty slices) on exactly sized heap
arrays: no access outside a tensor, no undefined index arithmetic, and the results satisfy
the adjoint identities and agree between the full loops and the element-wise routines."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = tmp_path / "oracle_sanitized"
    subprocess.check_call(["gcc", "-std=c11", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           "-fopenmp", "-Wall", "-Wextra", "-o", str(exe), os.path.join(ROOT, "oracle", "conv_oracle.c"),
                           os.path.join(ROOT, "tests", "oracle_sanitize_main.c"), "-lm"])
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1")
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=600, env=env)
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.startswith("ok "), r.stdout
