"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (CPU): the C source is built with
-fsanitize=address,undefined and the three pin files run against that build in a child process
(libasan is preloaded into the Python host; leak checking is off because the interpreter itself
never frees everything).  An out-of-bounds access, a use after free, a signed overflow, a
misaligned access or an invalid shift anywhere the pins reach aborts the child."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "adacomp_oracle.c")
PINS = ["tests/test_oracle_select.py", "tests/test_oracle_apply.py", "tests/test_oracle_wire.py"]


def _runtime(name):
    out = subprocess.run(["gcc", f"-print-file-name={name}"], capture_output=True, text=True).stdout.strip()
    return out if os.path.isabs(out) and os.path.exists(out) else None


def test_pins_pass_on_a_sanitized_build(tmp_path):
    asan, ubsan = _runtime("libasan.so"), _runtime("libubsan.so")
    if not asan:
        pytest.skip("gcc has no libasan here")
    lib = tmp_path / "liboracle_san.so"
    subprocess.run(["gcc", "-O1", "-g", "-std=gnu11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
                    SRC, "-lm", "-o", str(lib)], check=True)
    preload = asan + (":" + ubsan if ubsan else "")
    if os.environ.get("LD_PRELOAD"):     # whatever is preloaded already stays preloaded, after the sanitizer runtime
        preload += ":" + os.environ["LD_PRELOAD"]
    env = dict(os.environ, ADACOMP_ORACLE_LIB=str(lib), LD_PRELOAD=preload,
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=1:halt_on_error=1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([sys.executable, "-m", "pytest", *PINS, "-x", "-q", "-p", "no:cacheprovider"],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=1500)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "ERROR: AddressSanitizer" not in r.stderr and "runtime error:" not in r.stderr, tail
    assert " passed" in r.stdout.splitlines()[-1], tail
