"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer: one C program (tests/host/oracle_sanitized.c)
that includes the oracle's source and drives every entry point over small messages whose buffers have exactly the
size the calls may touch."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_touches_no_byte_outside_its_buffers(tmp_path):
    exe = tmp_path / "oracle_sanitized"
    subprocess.run(["gcc", "-std=c11", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-static-libasan", "-Wall", "-Wextra", "-Wno-unknown-pragmas", "-o", str(exe),
                    os.path.join(ROOT, "tests", "host", "oracle_sanitized.c"), "-lm"], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300, env=env)
    assert r.returncode == 0, (r.stdout + r.stderr)[-3000:]
    assert "oracle_sanitized: ok" in r.stdout
