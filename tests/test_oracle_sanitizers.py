"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: a C driver
(tests/oracle_sanitizer_driver.c) takes every entry point of the oracle through a tiny fp32
model and a tiny bf16 / grouped-query one -- computed and forced exits, a head subset, the
width bound at the largest width, eager alignment, sampling-mode rounds, rewind, single steps,
refused arguments -- and must finish without a report.  CPU only."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))


def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    subprocess.check_call(["gcc", "-std=gnu11", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           "-fopenmp", "-Wall", "-Wextra", "-Wno-unused-parameter",
                           os.path.join(HERE, "oracle_sanitizer_driver.c"), "-o", exe, "-lm"])
    env = dict(os.environ, OMP_NUM_THREADS="2", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "oracle sanitizer run: ok" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr


def test_oracle_float_build_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san32")
    subprocess.check_call(["gcc", "-std=gnu11", "-O1", "-g", "-DORC_F32", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", "-fopenmp", "-Wno-unused-parameter",
                           os.path.join(HERE, "oracle_sanitizer_driver.c"), "-o", exe, "-lm"])
    r = subprocess.run([exe], env=dict(os.environ, OMP_NUM_THREADS="2"), capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
