"""Sanitizer builds of the host-side C / C++ code: the CPU oracle and the length-balanced partitioner are compiled
under AddressSanitizer + UndefinedBehaviorSanitizer together with a small driver (tests/sanitize/) that calls every
entry point on ragged inputs with buffers of exactly the documented sizes.  A read or write past an array, a
misaligned access, signed overflow or a leak ends the driver with a non-zero status.  (GPU code has no sanitizer
here; its written buffers are covered by the guard-band test.)"""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-static-libasan",
       "-fno-omit-frame-pointer", "-Wall", "-Wextra"]


def _build_and_run(tmp_path, compiler, flags, sources, libs):
    exe = str(tmp_path / "check")
    cmd = [compiler, *flags, *SAN, *[os.path.join(ROOT, s) if not s.startswith("-") else s for s in sources],
           "-o", exe, *libs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0 and "asan" in r.stderr.lower() and "cannot find" in r.stderr.lower():
        pytest.skip("no static AddressSanitizer runtime for this compiler")
    assert r.returncode == 0, r.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="4")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), (r.stdout + r.stderr)[-3000:]


def test_oracle_under_address_and_ub_sanitizers(tmp_path):
    _build_and_run(tmp_path, "gcc", ["-std=c99", "-fopenmp"],
                   ["oracle/varlen_attn_oracle.c", "tests/sanitize/oracle_check.c"], ["-lm"])


def test_partitioner_under_address_and_ub_sanitizers(tmp_path):
    # va_partition.hip is pure host C++ (it includes only the C header)
    _build_and_run(tmp_path, "g++", ["-std=c++17"],
                   ["-xc++", "paper_2605_08962_amd/csrc/va_partition.hip", "tests/sanitize/partition_check.cc"], [])
