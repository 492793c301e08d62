"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only, no GPU).

oracle/gq_oracle.c and the driver tests/sanitize/oracle_driver.c are compiled together with
-fsanitize=address,undefined -fno-sanitize-recover=all and the driver is run as a subprocess.  The driver
calls every gqo_* function on ragged sizes (d = 0, 1, 31, 33, ...; K = 1 and 64; s at each storage format's
limit; coordinate offsets past 2^34; both draw widths; every random-word extreme; unusable norms; NaN, Inf,
denormal and negative-zero coordinates) with heap buffers of exactly the entitled size, so an access one
element too far, a signed overflow or a bad shift anywhere in the oracle fails this test.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE = os.path.join(ROOT, "oracle", "gq_oracle.c")
DRIVER = os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c")
# the oracle's own flags (single IEEE operations as written) plus the sanitizers; the run-time libraries are
# linked statically so that nothing preloaded into the process comes before them
CFLAGS = ["-std=c11", "-O1", "-g", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra", "-Werror",
          "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan"]


def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    exe = str(tmp_path / "oracle_driver")
    build = subprocess.run([gcc] + CFLAGS + ["-o", exe, ORACLE, DRIVER, "-lm"], stdout=subprocess.PIPE,
                           stderr=subprocess.STDOUT, text=True)
    assert build.returncode == 0, build.stdout
    env = dict(os.environ)
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    for leaks in ("1", "0"):
        env["ASAN_OPTIONS"] = "detect_leaks=%s:abort_on_error=0" % leaks
        run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
        # the leak checker needs ptrace, which some containers forbid: then the memory checks still count
        if leaks == "1" and "LeakSanitizer has encountered a fatal error" in run.stdout:
            continue
        break
    assert run.returncode == 0, run.stdout[-4000:]
    assert "0 failed checks" in run.stdout and "whole-path cases" in run.stdout
