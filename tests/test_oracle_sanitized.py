"""The oracle's pins once more, against a build of oracle/pqc_oracle.c instrumented with the address and the
undefined-behaviour sanitizers (host code, gcc): an out-of-bounds read, a signed overflow or a misaligned access in
the oracle would otherwise go unnoticed as long as the numbers come out right.  The instrumented library is loaded
through the oracle's PQC_ORACLE_LIB hook in a child process that runs tests/test_oracle_pins.py."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "pqc_oracle.c")


def _gcc_file(name: str) -> str:
    return subprocess.run(["gcc", f"-print-file-name={name}"], capture_output=True, text=True, check=True).stdout.strip()


@pytest.mark.timeout(900)
def test_pins_hold_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    lib = str(tmp_path / "libpqc_oracle_san.so")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off", "-mavx2", "-mfma",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           "-Wall", "-Wextra", "-shared", "-fPIC", SRC, "-o", lib, "-lm"]
    subprocess.run(cmd, check=True)
    asan = _gcc_file("libasan.so")
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("no address sanitizer runtime beside this gcc")
    env = dict(os.environ)
    # the sanitizer runtime must be the first library of the process (python itself is not instrumented); whatever is
    # preloaded already stays, behind it
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["PQC_ORACLE_LIB"] = lib
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:halt_on_error=1"  # the interpreter's own allocations are not the subject
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True)
    tail = (r.stdout + r.stderr)[-4000:]
    assert r.returncode == 0, "pins failed (or a sanitizer stopped the run) under the instrumented oracle:\n" + tail
    assert "passed" in r.stdout and "AddressSanitizer" not in tail and "runtime error" not in tail, tail
