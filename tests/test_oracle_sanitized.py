"""The oracle's pins once more against an AddressSanitizer + UndefinedBehaviorSanitizer
build of the same C source (CPU only).  The oracle is the ground truth of every parity
claim, so an out-of-bounds access, a use of freed memory or a signed overflow in it must
not go unnoticed.  The instrumented library is loaded into a child interpreter that runs
the pin file; the sanitizers abort that process on the first finding."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "moshpit_oracle.c")


def test_pins_pass_under_asan_and_ubsan(tmp_path):
    gcc = shutil.which("gcc")
    assert gcc, "gcc is needed to build the oracle"
    runtime = subprocess.check_output([gcc, "-print-file-name=libasan.so"], text=True).strip()
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("this gcc ships no AddressSanitizer runtime")
    lib = str(tmp_path / "libmoshpit_oracle_san.so")
    subprocess.check_call([gcc, "-O1", "-g", "-std=c11", "-Wall", "-Wextra", "-ffp-contract=off",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                           "-shared", "-fPIC", "-o", lib, SRC, "-lm"])
    env = dict(os.environ)
    env["MOSHPIT_ORACLE_LIB"] = lib
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # the interpreter itself is not instrumented: its allocations at exit are not leaks of the oracle
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    run = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                          "-x", "-q", "-p", "no:cacheprovider"], env=env, cwd=ROOT, capture_output=True, text=True,
                         timeout=900)
    tail = (run.stdout + run.stderr)[-4000:]
    assert run.returncode == 0, f"pins failed under the sanitizers:\n{tail}"
    assert " passed" in run.stdout and "AddressSanitizer" not in tail and "runtime error" not in tail
