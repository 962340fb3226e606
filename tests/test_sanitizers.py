"""AddressSanitizer + UndefinedBehaviorSanitizer runs of everything that executes on the host without a GPU:
the C oracle (gcc) and the host-only entry points of the library - argument validation, tile schedule,
speculative bookkeeping - compiled from the same source file as the product (hipcc, sanitizers on the host
side only).  The drivers in tests/sanitize/ keep every buffer in a heap block of its exact size."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _run(exe):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, env=env, timeout=600)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "ok" in res.stdout
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, res.stderr


def test_oracle_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=undefined", "-o", exe, os.path.join(SAN, "oracle_san.c"),
                           os.path.join(ROOT, "oracle", "nfd_oracle.c"), "-lm"])
    _run(exe)


@pytest.mark.skipif(shutil.which(HIPCC) is None, reason="hipcc not found")
def test_host_entry_points_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "host_san")
    cmd = [HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Wno-unused-value", "-Wno-inline-asm",
           "-o", exe, os.path.join(SAN, "host_san.cpp"),
           os.path.join(ROOT, "paper_2506_01380_amd", "csrc", "nfd_attn.hip")]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, cwd=str(tmp_path))
    assert res.returncode == 0, res.stdout
    _run(exe)
