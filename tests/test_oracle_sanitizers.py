"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): a copy of
oracle/co3_oracle.c is built with -fsanitize=address,undefined and all pin tests run against it in a child
process (CO3_ORACLE_LIB selects the library).  A report from either sanitizer aborts the child."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "co3_oracle.c")
PIN_FILES = ["tests/test_oracle_pins.py", "tests/test_oracle_bias_rule.py", "tests/test_oracle_layer_codes.py"]


def sanitizer_runtime():
    path = subprocess.run(["gcc", "-print-file-name=libasan.so"], stdout=subprocess.PIPE, text=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


@pytest.mark.skipif(sanitizer_runtime() is None, reason="gcc's AddressSanitizer runtime is not installed")
def test_pins_pass_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    so = str(tmp_path / "co3_oracle_san.so")
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
                           "-o", so, SRC, "-lm"])
    # the interpreter is not instrumented: the sanitizer runtime has to come first among the loaded libraries
    # (whatever else is preloaded stays, behind it); Python's own allocations are not this test's business
    preload = ":".join(x for x in (sanitizer_runtime(), os.environ.get("LD_PRELOAD", "")) if x)
    env = dict(os.environ, CO3_ORACLE_LIB=so, LD_PRELOAD=preload,
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=1:verify_asan_link_order=0",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([sys.executable, "-m", "pytest", *PIN_FILES, "-x", "-q", "-p", "no:cacheprovider"], cwd=ROOT, env=env,
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=1500)
    assert r.returncode == 0, r.stdout[-3000:]
    assert "AddressSanitizer" not in r.stdout and "runtime error" not in r.stdout, r.stdout[-3000:]
    assert " passed" in r.stdout
