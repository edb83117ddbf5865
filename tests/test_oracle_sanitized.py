"""The oracle's pins once more against a build of oracle/freeze_oracle.c with the address and
undefined-behaviour sanitizers (gcc -fsanitize=address,undefined): an out-of-bounds read, a use
after free, a signed overflow or a misaligned access anywhere in the checker fails this test.
Runs in a child process, because the sanitizer runtime has to be loaded before anything else."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_pins_pass_under_address_and_undefined_sanitizers():
    asan = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    assert os.path.isabs(asan) and os.path.exists(asan), "no sanitizer runtime next to gcc"
    env = dict(os.environ)
    env["FREEZE_ORACLE_SANITIZE"] = "1"
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # the interpreter and its extension modules are not built for leak checking; everything else stays on
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                          os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (res.stdout + res.stderr)[-3000:]
    assert res.returncode == 0, tail
    assert " passed" in res.stdout and "failed" not in res.stdout, tail
    assert "ERROR: AddressSanitizer" not in tail and "runtime error:" not in tail, tail
    assert os.path.exists(os.path.join(ROOT, "oracle", "libfreeze_oracle_san.so"))
