"""Host-side sanitizer runs (no GPU): the fp64 oracle and the argument-check layer of the C ABI,
each built with AddressSanitizer and UndefinedBehaviorSanitizer and driven by a small program
under tests/san/.  The sanitizer runtimes are linked into those programs, nothing is preloaded."""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "san")
ORACLE_C = os.path.join(ROOT, "oracle", "spo_oracle.c")
GCC = ["gcc", "-std=c11", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
       "-fno-omit-frame-pointer", "-fopenmp", "-ffp-contract=off"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
           OMP_NUM_THREADS="4")


def _build_oracle_driver(tmp_path, source):
    exe = str(tmp_path / "oracle_san")
    subprocess.run([*GCC, source, os.path.join(SAN, "oracle_san_driver.c"), "-o", exe, "-lm"], check=True)
    return exe


def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = _build_oracle_driver(tmp_path, ORACLE_C)
    r = subprocess.run([exe], capture_output=True, text=True, env=ENV, timeout=300)
    assert r.returncode == 0, r.stderr[-3000:]
    assert "oracle sanitizer run ok" in r.stdout


def test_a_planted_overrun_in_a_copy_of_the_oracle_is_caught(tmp_path):
    # the driver hands the oracle exact-size arrays: one logit too many must end the run
    src = open(ORACLE_C).read()
    planted, n = re.subn(r"for \(int64_t v = 0; v < V; \+\+v\) s \+= exp\(z\[v\] - c\);",
                         "for (int64_t v = 0; v <= V; ++v) s += exp(z[v] - c);", src)
    assert n == 1
    bad = tmp_path / "spo_oracle_planted.c"
    bad.write_text(planted)
    exe = _build_oracle_driver(tmp_path, str(bad))
    r = subprocess.run([exe], capture_output=True, text=True, env=ENV, timeout=300)
    assert r.returncode != 0 and "AddressSanitizer" in r.stderr


@pytest.mark.timeout(600)
def test_abi_argument_checks_run_clean_under_asan_and_ubsan(tmp_path):
    from paper_2509_13232_amd import build
    exe = build.build_sanitized_driver(os.path.join(SAN, "abi_san_driver.cpp"), str(tmp_path / "abi_san"))
    # the HIP runtime keeps allocations of its own until the process ends: leaks are not looked for here
    r = subprocess.run([exe], capture_output=True, text=True, env=dict(ENV, ASAN_OPTIONS="detect_leaks=0"), timeout=300)
    assert r.returncode == 0, (r.stdout + r.stderr)[-3000:]
    assert "ABI host-side sanitizer run ok" in r.stdout
