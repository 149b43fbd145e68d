"""The oracle's pins once more against a build of the oracle with the undefined-behaviour sanitizer
(shifts, signed overflow, misaligned or out-of-bounds accesses that the compiler can see) and with
bounds-checked fortified libc calls: a report aborts the run.  CPU only."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "ckks_oracle.c")


def test_oracle_pins_pass_under_the_undefined_behaviour_sanitizer(tmp_path):
    lib = tmp_path / "libckks_oracle_ubsan.so"
    subprocess.check_call(["gcc", "-O1", "-g", "-fopenmp", "-fPIC", "-shared", "-D_FORTIFY_SOURCE=2",
                           "-fsanitize=undefined", "-fno-sanitize-recover=all", "-o", str(lib), SRC])
    env = dict(os.environ, CKKS_ORACLE_LIB=str(lib), UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider", "-k",
                        "bigint or crt or level or rescale or merged or hoisted or bsgs or keyswitch or hmult or hrot"],
                       capture_output=True, text=True, env=env, cwd=ROOT)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
    assert "passed" in r.stdout and "runtime error" not in r.stderr
