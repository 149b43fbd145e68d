"""The oracle's pins once more against sanitizer builds of the oracle: the undefined-behaviour sanitizer (shifts,
signed overflow, misaligned accesses) and the address sanitizer (out-of-bounds and use-after-free accesses of the
C code on the arrays that numpy hands it), with bounds-checked fortified libc calls: a report aborts the run.
CPU only."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "ckks_oracle.c")
PINS = "bigint or crt or level or rescale or merged or hoisted or bsgs or keyswitch or hmult or hrot or ntt_batch or diagonals"


def _run_pins(env):
    return subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                           "-p", "no:cacheprovider", "-k", PINS], capture_output=True, text=True, env=env, cwd=ROOT)


def test_oracle_pins_pass_under_the_undefined_behaviour_sanitizer(tmp_path):
    lib = tmp_path / "libckks_oracle_ubsan.so"
    subprocess.check_call(["gcc", "-O1", "-g", "-fopenmp", "-fPIC", "-shared", "-D_FORTIFY_SOURCE=2",
                           "-fsanitize=undefined", "-fno-sanitize-recover=all", "-o", str(lib), SRC])
    r = _run_pins(dict(os.environ, CKKS_ORACLE_LIB=str(lib), UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1"))
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
    assert "passed" in r.stdout and "runtime error" not in r.stderr


def test_oracle_pins_pass_under_the_address_sanitizer(tmp_path):
    """The sanitizer runtime has to be in the process before the interpreter starts (the oracle is loaded through
    ctypes), hence LD_PRELOAD; leak checking is off because the interpreter itself never frees everything."""
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("no libasan in this toolchain")
    lib = tmp_path / "libckks_oracle_asan.so"
    subprocess.check_call(["gcc", "-O1", "-g", "-fopenmp", "-fPIC", "-shared", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-o", str(lib), SRC])
    preload = ":".join(x for x in (asan, os.environ.get("LD_PRELOAD", "")) if x)
    env = dict(os.environ, CKKS_ORACLE_LIB=str(lib), LD_PRELOAD=preload, OMP_NUM_THREADS="2",
               ASAN_OPTIONS="detect_leaks=0:halt_on_error=1:verify_asan_link_order=0:abort_on_error=0",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = _run_pins(env)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-3000:]
    assert "passed" in r.stdout and "AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr
