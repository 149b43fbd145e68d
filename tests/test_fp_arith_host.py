"""CPU check of the FP64 modular arithmetic of the HIP kernels (csrc/modarith.h, __host__ __device__).

x86-64 FMA and CDNA4 FMA are both IEEE-754 binary64, so exactness and range bounds shown on the host
carry over to the GPU.  The checker (tests/host/fparith_check.hip) is compiled with hipcc and run on the
CPU against 128-bit integer arithmetic: lazy products for inputs up to 8q, reductions, conversions, and
four-stage forward / inverse butterfly rounds from their documented start ranges.
"""
import os
import subprocess

import pytest

from paper_2310_16530_amd import synth

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.fixture(scope="module")
def checker(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("fpcheck") / "fparith_check")
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    subprocess.check_call([hipcc, "-O2", "-ffp-contract=off", "--offload-arch=gfx950", "-Xclang", "-target-feature",
                           "-Xclang", "-packed-fp32-ops", "-o", exe, os.path.join(HERE, "host", "fparith_check.hip")],
                          stderr=subprocess.DEVNULL)
    return exe


def test_fp64_arithmetic_is_exact_on_the_supported_range(checker):
    limit = 3 << 48  # primes strictly below this use the FP64 arithmetic
    moduli = [synth.CFG2.q_primes[0], synth.CFG4.q_primes[-1], synth.CFG0.q_primes[0], synth.CFG0.p_primes[0],
              limit - 1, limit - 7, 12289, (1 << 49) - 1]
    out = subprocess.run([checker] + [str(m) for m in moduli], capture_output=True, text=True, timeout=300)
    assert out.returncode == 0 and out.stdout.startswith("OK"), out.stdout + out.stderr
