"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: oracle/dsmoe_oracle.c is built
with -fsanitize=address,undefined together with a C driver (tests/csrc/sanitize_driver.c) that walks
the tiny brute-force grid with exactly sized buffers, and run in a child process.  Any report
(out-of-bounds access, use after free, leak, signed overflow, misaligned access ...) fails the test.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "sanitize_driver")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-Wall", "-Wextra", "-o", exe,
           os.path.join(HERE, "csrc", "sanitize_driver.c"), os.path.join(ROOT, "oracle", "dsmoe_oracle.c"), "-lm"]
    b = subprocess.run(cmd, capture_output=True, text=True)
    assert b.returncode == 0, b.stderr
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "abort_on_error=0:exitcode=23:detect_leaks=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    sys.stdout.write(r.stdout)
    assert r.returncode == 0, "sanitizer or check failure (exit %d):\n%s" % (r.returncode, r.stderr[-4000:])
    assert "sanitize_driver: ok" in r.stdout
    assert "runtime error" not in r.stderr and "ERROR: AddressSanitizer" not in r.stderr and "LeakSanitizer" not in r.stderr
