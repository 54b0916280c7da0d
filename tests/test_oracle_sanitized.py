"""The oracle's C code under AddressSanitizer and UndefinedBehaviorSanitizer (host only).

``oracle/dlrt_oracle.c`` and the driver beside this file are compiled together with
``-fsanitize=address,undefined``; the driver calls every oracle function on exactly-sized heap buffers over
small and ragged shapes, so any read or write outside a buffer, signed overflow or misaligned access ends the
run with a report and a non-zero status.
"""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitized")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-omit-frame-pointer",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-Wall", "-Wextra",
           os.path.join(ROOT, "oracle", "dlrt_oracle.c"), os.path.join(ROOT, "tests", "oracle_sanitizer_driver.c"),
           "-o", exe, "-lm"]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    env = dict(os.environ, OMP_NUM_THREADS="2", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0")
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-3000:]
    assert r.stdout.startswith("checksum ")
