"""AddressSanitizer + UndefinedBehaviorSanitizer over the CPU oracle (host code only: GPU sanitizers are not
available).  ``tests/sanitize_oracle_main.c`` includes ``oracle/mars_ref.c`` and drives every exported function
on 180 seeded cases; the sanitizers abort on the first out-of-bounds access, signed overflow or misaligned
access.  A finding here is a finding in the checker every parity test trusts."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = tmp_path / "sanitize_oracle"
    build = subprocess.run(["gcc", "-O1", "-g", "-std=c99", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                            "-fno-omit-frame-pointer", "-Wall", "-o", str(exe),
                            os.path.join(HERE, "sanitize_oracle_main.c"), "-lm"], capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-2000:]
    env = dict(os.environ)
    # another library may already be preloaded into every process: the sanitizer runtime then is not the first in
    # the list, which it only checks for by default; leak checking needs ptrace, which containers often deny
    env["ASAN_OPTIONS"] = "verify_asan_link_order=0:detect_leaks=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    run = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=600)
    assert run.returncode == 0, (run.stdout[-1000:], run.stderr[-3000:])
    assert "180 cases, 0 failed" in run.stdout, run.stdout
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr[-3000:]
