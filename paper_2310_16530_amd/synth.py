"""Seeded synthetic inputs and parameter sets for the RNS-CKKS key-switch path.

This module is the only code shared by the HIP path, the CPU oracle, the tests
and the benchmark.  It holds NO arithmetic of the method (no NTT, no base
conversion, no key generation): it only
  * chooses the RNS prime chains (smallest primes above a power of two that
    are congruent to 1 modulo 2N),
  * names the five workload shapes, and
  * draws the random numbers (uniform residues, ternary secrets, rounded
    Gaussian errors) from a seeded numpy generator.
Polynomials follow the paper's Section 2 object: an L x N integer matrix stored
limb-major as uint64 words.
"""
from __future__ import annotations

from dataclasses import dataclass
from functools import lru_cache
from typing import List, Sequence, Tuple

import numpy as np

SEED_BASE = 0xC0FFEE00
SIGMA = 3.2
GAUSS_CUT = 19  # 6 sigma


# --------------------------------------------------------------------------
# prime chains
# --------------------------------------------------------------------------
_MR_BASES = (2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37)


def is_prime(n: int) -> bool:
    """Deterministic Miller-Rabin for n < 3.3e24 (bases 2..37)."""
    if n < 2:
        return False
    for p in _MR_BASES:
        if n % p == 0:
            return n == p
    d, r = n - 1, 0
    while d % 2 == 0:
        d //= 2
        r += 1
    for a in _MR_BASES:
        x = pow(a, d, n)
        if x == 1 or x == n - 1:
            continue
        for _ in range(r - 1):
            x = x * x % n
            if x == n - 1:
                break
        else:
            return False
    return True


@lru_cache(maxsize=None)
def primes_above(bound: int, two_n: int, count: int) -> Tuple[int, ...]:
    """The `count` smallest primes p > bound with p = 1 (mod two_n)."""
    out: List[int] = []
    c = bound - (bound % two_n) + 1
    while c <= bound:
        c += two_n
    while len(out) < count:
        if is_prime(c):
            out.append(c)
        c += two_n
    return tuple(out)


@dataclass(frozen=True)
class ParamSet:
    """One RNS-CKKS parameter set: ring degree, q-limbs, special limbs, digits."""
    name: str
    logN: int
    L: int
    K: int
    dnum: int
    q_floor_bits: int  # q-limbs are the L smallest primes above 2**q_floor_bits
    p_floor_bits: int  # special limbs are the K smallest primes above 2**p_floor_bits

    @property
    def N(self) -> int:
        return 1 << self.logN

    @property
    def alpha(self) -> int:
        return -(-self.L // self.dnum)  # the last digit is shorter when dnum does not divide L

    @property
    def q_primes(self) -> Tuple[int, ...]:
        return primes_above(1 << self.q_floor_bits, 2 * self.N, self.L)

    @property
    def p_primes(self) -> Tuple[int, ...]:
        if self.K == 0:
            return ()
        return primes_above(1 << self.p_floor_bits, 2 * self.N, self.K)

    @property
    def primes(self) -> Tuple[int, ...]:
        """Prime order used everywhere: q_0..q_{L-1}, p_0..p_{K-1}."""
        return self.q_primes + self.p_primes


@dataclass(frozen=True)
class ExplicitParamSet:
    """A parameter set given by its primes (same attributes as ParamSet), for chains that mix prime sizes."""
    name: str
    logN: int
    dnum: int
    q_primes: Tuple[int, ...]
    p_primes: Tuple[int, ...]

    @property
    def N(self) -> int:
        return 1 << self.logN

    @property
    def L(self) -> int:
        return len(self.q_primes)

    @property
    def K(self) -> int:
        return len(self.p_primes)

    @property
    def alpha(self) -> int:
        return -(-self.L // self.dnum)  # the last digit is shorter when dnum does not divide L

    @property
    def primes(self) -> Tuple[int, ...]:
        return self.q_primes + self.p_primes


def mixed_params(logN: int, q_floors: Sequence[int], p_floors: Sequence[int], dnum: int,
                 name: str = "mixed") -> ExplicitParamSet:
    """Limb i is the next unused prime = 1 mod 2N above floor i; a floor below 64 means 2**floor."""
    used: List[int] = []

    def pick(floor: int) -> int:
        bound = (1 << floor) if floor < 64 else floor
        k = 1
        while True:
            cand = primes_above(bound, 2 << logN, k)[-1]
            if cand not in used:
                used.append(cand)
                return cand
            k += 1

    q = tuple(pick(f) for f in q_floors)
    pp = tuple(pick(f) for f in p_floors)
    return ExplicitParamSet(name, logN, dnum, q, pp)


# The five workload shapes (workloads 0..4 of the benchmark definition).
CFG0 = ParamSet("cfg0_hmult_n12", 12, 3, 1, 3, 35, 36)
CFG1 = ParamSet("cfg1_ntt_n16_l24", 16, 24, 0, 1, 49, 59)
CFG2 = ParamSet("cfg2_hmult_n16_l24_d4", 16, 24, 6, 4, 49, 59)
CFG3 = ParamSet("cfg3_rotsum_n16_l24_d4", 16, 24, 6, 4, 49, 59)
CFG4 = ParamSet("cfg4_cts_n16_l35_d5", 16, 35, 7, 5, 49, 59)
CONFIGS = (CFG0, CFG1, CFG2, CFG3, CFG4)

CFG1_BATCH = 16
CFG2_BATCH = 8
# configs[3] lists 17 offsets while calling them 16; the list is kept as given.
CFG3_ROTATIONS = tuple(range(1, 9)) + tuple(1 << i for i in range(4, 12)) + (-1,)
# configs[4]: +-2^i for i = 0..15 (32 jobs; +-2^15 is the identity on 2^15 slots).
CFG4_ROTATIONS = tuple(s * (1 << i) for i in range(16) for s in (1, -1))


def small_params(logN: int, L: int, K: int, dnum: int, q_floor_bits: int = 49,
                 p_floor_bits: int = 59, name: str = "small") -> ParamSet:
    """A reduced shape of the same family, for parity cases the oracle finishes fast."""
    return ParamSet(name, logN, L, K, dnum, q_floor_bits, p_floor_bits)


def galois_element(rotation: int, logN: int) -> int:
    """Slot rotation r -> Galois element 5^(r mod N/2) mod 2N."""
    n = 1 << logN
    return pow(5, rotation % (n // 2), 2 * n)


# --------------------------------------------------------------------------
# seeded random draws
# --------------------------------------------------------------------------
def rng_for(config_index: int, stream: int = 0) -> np.random.Generator:
    """Independent generator per (config, buffer)."""
    return np.random.Generator(np.random.Philox(key=SEED_BASE + config_index, counter=[0, 0, 0, stream]))


def uniform_residues(rng: np.random.Generator, primes: Sequence[int], n: int,
                     lead: Tuple[int, ...] = ()) -> np.ndarray:
    """uint64 array lead + (len(primes), n); row i uniform in [0, primes[i])."""
    out = np.empty(tuple(lead) + (len(primes), n), dtype=np.uint64)
    for i, p in enumerate(primes):
        out[..., i, :] = rng.integers(0, p, size=tuple(lead) + (n,), dtype=np.uint64)
    return out


def ternary_iid(rng: np.random.Generator, n: int) -> np.ndarray:
    """int8 secret, coefficients iid uniform on {-1, 0, 1}."""
    return rng.integers(-1, 2, size=n, dtype=np.int8)


def ternary_hamming(rng: np.random.Generator, n: int, weight: int) -> np.ndarray:
    """int8 secret with exactly `weight` non-zeros at distinct uniform positions, signs iid."""
    s = np.zeros(n, dtype=np.int8)
    pos = rng.choice(n, size=weight, replace=False)
    s[pos] = rng.integers(0, 2, size=weight, dtype=np.int8) * 2 - 1
    return s


def gaussian_error(rng: np.random.Generator, shape) -> np.ndarray:
    """int64 errors: round-to-nearest of N(0, 3.2^2), resampled while |e| > 19."""
    e = np.rint(rng.normal(0.0, SIGMA, size=shape)).astype(np.int64)
    bad = np.abs(e) > GAUSS_CUT
    while bad.any():
        e[bad] = np.rint(rng.normal(0.0, SIGMA, size=int(bad.sum()))).astype(np.int64)
        bad = np.abs(e) > GAUSS_CUT
    return e
