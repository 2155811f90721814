"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: tests/sanitize/driver.c feeds its
decoders thousands of corrupted streams (every header bit, random plane bits, truncations, short capacities).
Host code only; needs no GPU."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_decoders_survive_corrupt_streams_under_sanitizers(tmp_path):
    exe = tmp_path / "oracle_san"
    subprocess.run(["gcc", "-std=c99", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-static-libasan", "-ffp-contract=off", "-o", str(exe),
                    os.path.join(ROOT, "oracle", "fastsgd_ref.c"), os.path.join(ROOT, "tests", "sanitize", "driver.c"), "-lm"],
                   check=True)
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert "sanitized runs:" in r.stdout and int(r.stdout.split(":")[1]) > 10000
