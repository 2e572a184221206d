"""The library's host layer (csrc/api.hip: validation, workspace carving, chunk loops, pointer arithmetic) compiled with
a plain host compiler under -fsanitize=address,undefined against stub kernel launchers that touch the ends of every
operand extent, and run over exactly sized allocations - at small ragged shapes and at the benchmark's shapes (CPU only,
no GPU, no HIP runtime).  A planted off-by-one must be reported."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "tests", "host_sanitize")


@pytest.fixture(scope="module")
def binary(tmp_path_factory):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no host C++ compiler")
    out = str(tmp_path_factory.mktemp("host_sanitize") / "host_sanitize")
    cmd = [gxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-I", SRC, "-I", os.path.join(ROOT, "paper_2506_03077_amd", "csrc"),
           "-x", "c++", os.path.join(ROOT, "paper_2506_03077_amd", "csrc", "api.hip"),
           os.path.join(SRC, "stub_launch.cpp"), os.path.join(SRC, "main.cpp"), "-o", out]
    p = subprocess.run(cmd, capture_output=True, text=True)
    assert p.returncode == 0, p.stderr[-4000:]
    return out


def run(binary, *args):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)          # the sanitizer runtime must come first in the library list
    return subprocess.run([binary, *args], capture_output=True, text=True, env=env, timeout=600)


def test_host_layer_is_clean_under_sanitizers_at_small_ragged_shapes(binary):
    p = run(binary)
    assert p.returncode == 0 and p.stdout.strip().startswith("OK: 0 failing cases"), (p.stdout[-2000:], p.stderr[-4000:])
    assert "runtime error" not in p.stderr and "AddressSanitizer" not in p.stderr


def test_host_layer_is_clean_under_sanitizers_at_the_benchmark_shapes(binary):
    p = run(binary, "big")
    assert p.returncode == 0 and p.stdout.strip().startswith("OK: 0 failing cases"), (p.stdout[-2000:], p.stderr[-4000:])
    assert "runtime error" not in p.stderr and "AddressSanitizer" not in p.stderr


def test_a_planted_short_buffer_is_reported(binary):
    p = run(binary, "planted")
    assert p.returncode != 0 and "heap-buffer-overflow" in p.stderr
