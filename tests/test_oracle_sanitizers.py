"""The C oracle built with AddressSanitizer and UndefinedBehaviorSanitizer (CPU only) and driven over
every entry point on exactly-sized heap buffers: a read or write outside an operand, a signed overflow
or a misaligned access inside the oracle ends the driver with a sanitizer report and a non-zero status."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitized")
    cmd = ["gcc", "-std=c11", "-O1", "-g", "-fno-omit-frame-pointer", "-ffp-contract=off",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           "-Wall", "-Wextra", "-o", exe,
           os.path.join(HERE, "oracle_sanitizer_driver.c"), os.path.join(ROOT, "oracle", "pg_oracle.c"), "-lm"]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "oracle sanitizer driver: ok" in res.stdout
