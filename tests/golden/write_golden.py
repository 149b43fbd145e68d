"""Regenerate prime_chains.txt and min_psi.txt.  Calls only the input module and the CPU oracle."""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2310_16530_amd import synth  # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))


def offsets(primes, bits, logn):
    return " ".join(str((p - (1 << bits) - 1) >> (logn + 1)) for p in primes)


def main():
    with open(os.path.join(HERE, "prime_chains.txt"), "w") as f:
        f.write("# name  logN  base_bits  offsets c (prime = 2^base_bits + c*2^(logN+1) + 1)\n")
        f.write("cfg0_q 12 35 %s\n" % offsets(synth.CFG0.q_primes, 35, 12))
        f.write("cfg0_p 12 36 %s\n" % offsets(synth.CFG0.p_primes, 36, 12))
        f.write("n16_q  16 49 %s\n" % offsets(synth.CFG4.q_primes, 49, 16))
        f.write("n16_p  16 59 %s\n" % offsets(synth.CFG4.p_primes, 59, 16))
    with open(os.path.join(HERE, "min_psi.txt"), "w") as f:
        f.write("# prime  logN  smallest psi with psi^N = -1 mod prime\n")
        for p in synth.CFG0.primes:
            f.write("%d 12 %d\n" % (p, oracle.min_psi(p, 12)))
        for p in (synth.CFG2.q_primes[0], synth.CFG2.p_primes[0]):
            f.write("%d 16 %d\n" % (p, oracle.min_psi(p, 16)))


if __name__ == "__main__":
    main()
