"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: a C driver (tests/oracle_sanitize_main.c)
calls every entry point on small seeded inputs with the edge cases in; the sanitized build must run clean and
print the checksums of the plain build.  No GPU."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = [os.path.join(ROOT, "oracle", "aasd_oracle.c"), os.path.join(ROOT, "tests", "oracle_sanitize_main.c")]


def _build(tmp_path, name, flags):
    exe = str(tmp_path / name)
    subprocess.check_call(["gcc", "-std=c11", "-g", "-Wall", "-Wextra", *flags, "-I", os.path.join(ROOT, "oracle"), "-o", exe, *SRC, "-lm"])
    return exe


def test_oracle_runs_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    plain = _build(tmp_path, "plain", ["-O2"])
    try:
        san = _build(tmp_path, "san", ["-O1", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                                       "-fno-sanitize-recover=all", "-static-libasan"])
    except subprocess.CalledProcessError:
        pytest.skip("this gcc has no sanitizer runtime")
    env = dict(os.environ)   # the runtime is linked statically into the driver, so the order of preloaded libraries does not matter to it
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    want = subprocess.run([plain], capture_output=True, text=True, check=True).stdout
    got = subprocess.run([san], capture_output=True, text=True, env=env)
    assert got.returncode == 0, got.stderr[-4000:]
    assert got.stdout == want and want.count("\n") >= 25
    assert "6627e8d5 e169c58d bc57ac4c 9b00dbd8" in want      # the driver does call the oracle: Philox known answer
