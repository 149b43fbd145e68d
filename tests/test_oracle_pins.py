"""Pins of the CPU oracle to things other than itself (runs without a GPU).

Root of trust: Python big integers -- schoolbook negacyclic products, CRT
reconstruction, direct polynomial substitution -- plus algebraic identities and
the decrypt-and-bound noise check.  A dropped term, wrong sign/index or a
transposed operand anywhere in oracle/ckks_oracle.c fails at least one of them.
"""
import os
import random

import numpy as np
import pytest

from paper_2310_16530_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def brev(x, bits):
    return int(format(x, "0%db" % bits)[::-1], 2) if bits else 0


def negacyclic_schoolbook(a, b, m):
    n = len(a)
    out = [0] * n
    for i, ai in enumerate(a):
        for j, bj in enumerate(b):
            k = i + j
            if k < n:
                out[k] = (out[k] + ai * bj) % m
            else:
                out[k - n] = (out[k - n] - ai * bj) % m
    return out


def crt(residues, moduli):
    M = 1
    for m in moduli:
        M *= m
    x = 0
    for r, m in zip(residues, moduli):
        Mi = M // m
        x += int(r) * Mi * pow(Mi, -1, m)
    return x % M, M


# --------------------------------------------------------------------- scalars
def test_modular_scalars_vs_bigint(orc):
    rnd = random.Random(1)
    mods = [17, 97, 34359754753, 2**49 + 13 * 2**17 + 1, 2**59 + 37 * 2**17 + 1, 2**62 + 135]
    for m in mods:
        edge = [0, 1, 2, m - 1, m - 2, m // 2, (1 << 59) % m, (1 << 32) % m]
        vals = edge + [rnd.randrange(m) for _ in range(40)]
        for a in vals:
            for b in vals[:12]:
                assert orc.mulmod(a, b, m) == a * b % m
                assert int(orc.lib().orc_addmod(a, b, m)) == (a + b) % m
                assert int(orc.lib().orc_submod(a, b, m)) == (a - b) % m
        for a in vals[1:20]:
            if a % m:
                assert orc.powmod(a, 12345, m) == pow(a, 12345, m)
    for m in [17, 97, 34359754753, 2**49 + 13 * 2**17 + 1]:
        for a in [1, 2, 3, m - 1, 12345 % m or 5]:
            assert orc.invmod(a, m) * a % m == 1


# ------------------------------------------------------------------ parameters
def test_prime_chains_match_golden():
    chains = {}
    for line in open(os.path.join(GOLD, "prime_chains.txt")):
        if line.startswith("#") or not line.strip():
            continue
        f = line.split()
        logn, bits = int(f[1]), int(f[2])
        chains[f[0]] = [2**bits + int(c) * 2**(logn + 1) + 1 for c in f[3:]]
    assert list(synth.CFG0.q_primes) == chains["cfg0_q"] == [34359754753, 34359771137, 34359795713]
    assert list(synth.CFG0.p_primes) == chains["cfg0_p"] == [68719484929]
    assert list(synth.CFG4.q_primes) == chains["n16_q"]
    assert list(synth.CFG4.p_primes) == chains["n16_p"]
    assert list(synth.CFG2.q_primes) == chains["n16_q"][:24]
    assert list(synth.CFG2.p_primes) == chains["n16_p"][:6]
    assert list(synth.CFG1.primes) == chains["n16_q"][:24]
    # smallest-above property, checked by exhaustive trial division on the small chain
    for p in synth.CFG0.primes:
        assert all(p % d for d in range(3, 1 << 19, 2))
    # P > Q_j in every set with special primes
    for ps in (synth.CFG0, synth.CFG2, synth.CFG4):
        P = np.prod([int(x) for x in ps.p_primes], dtype=object)
        for j in range(ps.dnum):
            Qj = np.prod([int(x) for x in ps.q_primes[j * ps.alpha:(j + 1) * ps.alpha]], dtype=object)
            assert P > Qj


def test_n16_chains_against_an_independent_primality_test():
    """The N = 2^16 chains are 'the smallest primes above 2^49 / 2^59 congruent to 1 mod 2^17': every member is
    prime and every smaller candidate of that form is composite, by sympy's primality test (not the generator's
    own Miller-Rabin, which also wrote the golden file)."""
    sympy = pytest.importorskip("sympy")
    step = 1 << 17
    for chain, floor in ((synth.CFG4.q_primes, 1 << 49), (synth.CFG4.p_primes, 1 << 59)):
        chain = [int(p) for p in chain]
        assert chain == sorted(chain) and len(set(chain)) == len(chain)
        members = set(chain)
        c = floor + 1
        while c <= chain[-1]:
            assert sympy.isprime(c) == (c in members), c
            c += step
    for p in synth.CFG0.primes:
        assert sympy.isprime(int(p))


def test_ntt_batch_maps_row_to_prime_and_matches_the_definition(orc):
    """Batched transform, batch 3 x 5 limbs (limb l of every polynomial uses prime l of the chain): every row
    against the big-integer definition, both directions."""
    logn, n = 5, 32
    ps = synth.small_params(logn, 3, 2, 3, 30, 31)
    P = orc.Params.from_set(ps)
    rng = np.random.default_rng(77)
    x = synth.uniform_residues(rng, ps.primes, n, lead=(3,))
    assert x.shape == (3, 5, n)
    fwd = orc.ntt_batch(x, P, 0)
    inv = orc.ntt_batch(fwd, P, 0, inverse=True)
    assert np.array_equal(inv, x)
    for b in range(3):
        for l in range(5):
            m, psi = int(ps.primes[l]), int(P.psi[l])
            row = [int(v) for v in x[b, l]]
            want = [sum(row[t] * pow(psi, t * (2 * brev(j, logn) + 1), m) for t in range(n)) % m for j in range(n)]
            assert fwd[b, l].tolist() == want, (b, l)
    # a sub-range of the chain: limbs 2..4 with prime_first = 2
    sub = np.ascontiguousarray(x[:, 2:5])
    assert np.array_equal(orc.ntt_batch(sub, P, 2), fwd[:, 2:5])


def test_min_psi_matches_golden_and_is_minimal(orc):
    for line in open(os.path.join(GOLD, "min_psi.txt")):
        if line.startswith("#") or not line.strip():
            continue
        m, logn, psi = (int(x) for x in line.split())
        got = orc.min_psi(m, logn)
        assert got == psi
        assert pow(psi, 1 << logn, m) == m - 1
    # brute-force minimality on small primes: no smaller element is a primitive 2N-th root
    for m, logn in [(17, 3), (97, 4), (193, 5), (257, 7), (12289, 11)]:
        n = 1 << logn
        brute = next(x for x in range(2, m) if pow(x, n, m) == m - 1)
        assert orc.min_psi(m, logn) == brute


# ------------------------------------------------------------------ transforms
TINY = [(17, 2), (17, 3), (97, 3), (97, 4), (193, 5), (257, 6), (257, 7), (12289, 6),
        (34359754753, 4), (2**49 + 13 * 2**17 + 1, 6), (2**59 + 37 * 2**17 + 1, 5)]


@pytest.mark.parametrize("m,logn", TINY)
def test_ntt_equals_bigint_definition(orc, m, logn):
    n = 1 << logn
    psi = orc.min_psi(m, logn)
    rnd = random.Random(m + logn)
    x = [rnd.randrange(m) for _ in range(n)]
    want = [sum(x[t] * pow(psi, t * (2 * brev(j, logn) + 1), m) for t in range(n)) % m for j in range(n)]
    xs = np.array(x, dtype=np.uint64)
    assert orc.ntt(xs, logn, m, psi).tolist() == want
    assert orc.ntt_def(xs, logn, m, psi).tolist() == want
    assert orc.intt(np.array(want, dtype=np.uint64), logn, m, psi).tolist() == x


@pytest.mark.parametrize("m,logn", [(257, 7), (12289, 8), (34359754753, 8), (2**49 + 13 * 2**17 + 1, 8),
                                    (2**59 + 37 * 2**17 + 1, 7)])
def test_ntt_multiply_equals_schoolbook_negacyclic(orc, m, logn):
    n = 1 << logn
    psi = orc.min_psi(m, logn)
    rnd = random.Random(7 * m + logn)
    a = [rnd.randrange(m) for _ in range(n)]
    b = [rnd.randrange(m) for _ in range(n)]
    A = orc.ntt(np.array(a, dtype=np.uint64), logn, m, psi)
    B = orc.ntt(np.array(b, dtype=np.uint64), logn, m, psi)
    C = np.array([int(x) * int(y) % m for x, y in zip(A, B)], dtype=np.uint64)
    assert orc.intt(C, logn, m, psi).tolist() == negacyclic_schoolbook(a, b, m)


def test_ntt_multiply_sampled_coefficients_n4096(orc):
    m, logn = synth.CFG0.q_primes[1], 12
    n = 1 << logn
    psi = orc.min_psi(m, logn)
    rng = np.random.default_rng(5)
    a = rng.integers(0, m, n, dtype=np.uint64)
    b = rng.integers(0, m, n, dtype=np.uint64)
    C = orc.pointwise("mul", orc.ntt(a, logn, m, psi)[None], orc.ntt(b, logn, m, psi)[None], [m])[0]
    c = orc.intt(C, logn, m, psi)
    al, bl = [int(v) for v in a], [int(v) for v in b]
    for k in [0, 1, 2, 77, 2047, 2048, 4094, 4095]:
        want = 0
        for i in range(n):
            j = k - i
            if j >= 0:
                want += al[i] * bl[j]
            else:
                want -= al[i] * bl[j + n]
        assert int(c[k]) == want % m


@pytest.mark.parametrize("logn", [10, 12, 16])
def test_ntt_closed_forms_and_roundtrip(orc, logn):
    n = 1 << logn
    for m in (synth.primes_above(1 << 49, 2 * n, 1)[0], synth.primes_above(1 << 59, 2 * n, 1)[0]):
        psi = orc.min_psi(m, logn)
        one = np.zeros(n, dtype=np.uint64)
        one[0] = 1
        assert (orc.ntt(one, logn, m, psi) == 1).all()          # NTT(1) = all ones
        X = np.zeros(n, dtype=np.uint64)
        X[1] = 1
        got = orc.ntt(X, logn, m, psi)                           # NTT(X)[j] = psi^(2 brev(j) + 1)
        for j in [0, 1, 2, 3, n // 2, n - 2, n - 1, 12345 % n]:
            assert int(got[j]) == pow(psi, 2 * brev(j, logn) + 1, m)
        rng = np.random.default_rng(logn)
        x = rng.integers(0, m, n, dtype=np.uint64)
        xh = orc.ntt(x, logn, m, psi)
        assert np.array_equal(orc.intt(xh, logn, m, psi), x)
        for j in [0, 1, n // 3, n - 1]:                          # fast network vs definition, sampled
            assert orc.ntt_def_at(x, logn, m, psi, j) == int(xh[j])
        # linearity with a big-int check of one slot
        y = rng.integers(0, m, n, dtype=np.uint64)
        s = orc.pointwise("add", x[None], y[None], [m])[0]
        assert np.array_equal(orc.ntt(s, logn, m, psi), orc.pointwise("add", xh[None], orc.ntt(y, logn, m, psi)[None], [m])[0])


def test_ntt_def_c_vs_fast_n1024(orc):
    m, logn = 2**59 + 37 * 2**17 + 1, 10
    psi = orc.min_psi(m, logn)
    x = np.random.default_rng(3).integers(0, m, 1 << logn, dtype=np.uint64)
    assert np.array_equal(orc.ntt_def(x, logn, m, psi), orc.ntt(x, logn, m, psi))


# ------------------------------------------------------------- base conversion
def _small_set(logn=5, L=4, K=2, dnum=2, qb=20, pb=24):
    return synth.small_params(logn, L, K, dnum, qb, pb)


@pytest.mark.parametrize("shape", [(5, 4, 2, 2, 20, 24), (4, 6, 3, 2, 20, 22), (4, 3, 1, 3, 35, 36),
                                   (3, 6, 6, 1, 30, 31), (4, 8, 2, 4, 49, 59), (4, 12, 3, 1, 49, 59), (3, 20, 10, 2, 30, 31),
                                   (4, 5, 2, 2, 20, 24), (4, 7, 3, 3, 35, 36), (3, 10, 4, 4, 49, 59)])
def test_modup_vs_bigint_crt(orc, shape):
    ps = _small_set(*shape)
    P = orc.Params.from_set(ps)
    rng = np.random.default_rng(11)
    x = synth.uniform_residues(rng, ps.q_primes, ps.N)
    # plant edge values
    x[:, 0] = 0
    for i, q in enumerate(ps.q_primes):
        x[i, 1] = q - 1
    out = orc.modup(x, P)
    assert out.shape == (ps.dnum, ps.L + ps.K, ps.N)
    a = ps.alpha
    for j in range(ps.dnum):
        digit = list(ps.q_primes[j * a:(j + 1) * a])              # the last digit is shorter when dnum does not divide L
        assert 1 <= len(digit) <= a
        for n in range(ps.N):
            xi, Qj = crt([x[j * a + i, n] for i in range(len(digit))], digit)
            us = set()
            for t, b in enumerate(ps.primes):
                if j * a <= t < j * a + len(digit):
                    assert out[j, t, n] == x[t, n]              # own limbs copied
                    continue
                diff = (int(out[j, t, n]) - xi) % b
                u = diff * pow(Qj, -1, b) % b
                us.add(u)
            assert len(us) == 1 and 0 <= us.pop() < len(digit)  # one common overflow u < digit size
            if len(digit) == 1:
                for t, b in enumerate(ps.primes):
                    assert int(out[j, t, n]) == xi % b           # alpha = 1: plain reduction


def test_conv_matches_termwise_bigint(orc):
    src = [1048609 + 0, 1049089, 1050113]
    src = list(synth.primes_above(1 << 20, 64, 3))
    b = synth.primes_above(1 << 24, 64, 1)[0]
    rng = np.random.default_rng(2)
    x = synth.uniform_residues(rng, src, 32)
    got = orc.conv(x, src, b)
    S = src[0] * src[1] * src[2]
    for n in range(32):
        want = 0
        for i, q in enumerate(src):
            hat = S // q
            y = int(x[i, n]) * pow(hat, -1, q) % q
            want += y * (hat % b)
        assert int(got[n]) == want % b


@pytest.mark.parametrize("shape", [(5, 4, 2, 2, 20, 24), (4, 6, 3, 2, 20, 22), (4, 3, 1, 3, 35, 36), (4, 8, 2, 4, 49, 59),
                                   (4, 3, 12, 1, 49, 59)])
def test_moddown_vs_bigint(orc, shape):
    ps = _small_set(*shape)
    P = orc.Params.from_set(ps)
    rng = np.random.default_rng(13)
    x = synth.uniform_residues(rng, ps.primes, ps.N)
    Pp = 1
    for p in ps.p_primes:
        Pp *= p
    Q = 1
    for q in ps.q_primes:
        Q *= q
    # coefficient 0: an exact multiple of P, whose special limbs are all zero -> exact division
    big = (rng.integers(0, 2**62, dtype=np.uint64).item() * 987654321987654321 % Q) * Pp
    for t, m in enumerate(ps.primes):
        x[t, 0] = big % m
    out = orc.moddown(x, P)
    for n in range(ps.N):
        c, PQ = crt([x[t, n] for t in range(ps.L + ps.K)], list(ps.primes))
        us = set()
        for i, q in enumerate(ps.q_primes):
            us.add((c // Pp - int(out[i, n])) % q)
        assert len(us) == 1
        u = us.pop()
        assert 0 <= u < ps.K
        if n == 0:
            assert u == 0 and all(int(out[i, 0]) == (big // Pp) % q for i, q in enumerate(ps.q_primes))


# ---------------------------------------------------------------- automorphism
def test_automorphism_coeff_by_substitution_and_eval_consistency(orc):
    for m, logn in [(97, 3), (257, 5), (2**49 + 13 * 2**17 + 1, 6)]:
        n = 1 << logn
        psi = orc.min_psi(m, logn)
        rnd = random.Random(m)
        x = [rnd.randrange(m) for _ in range(n)]
        xs = np.array(x, dtype=np.uint64)
        for g in [1, 3, 5, 25 % (2 * n), pow(5, -1, 2 * n), 2 * n - 1]:
            want = [0] * n                                     # substitute X -> X^g, reduce by X^n = -1
            for t, c in enumerate(x):
                e = t * g
                sign = -1 if (e // n) % 2 else 1
                want[e % n] = (want[e % n] + sign * c) % m
            got = orc.automorph_coeff(xs, logn, m, g)
            assert got.tolist() == want
            lhs = orc.ntt(got, logn, m, psi)                   # NTT(sigma(x)) = sigma_eval(NTT(x))
            rhs = orc.automorph_eval(orc.ntt(xs, logn, m, psi), logn, g)
            assert np.array_equal(lhs, rhs)
            ginv = pow(g, -1, 2 * n)
            assert np.array_equal(orc.automorph_coeff(got, logn, m, ginv), xs)
            assert np.array_equal(orc.automorph_eval(rhs, logn, ginv), orc.ntt(xs, logn, m, psi))
        assert np.array_equal(orc.automorph_coeff(xs, logn, m, 1), xs)
        # multiplicativity on evaluation form
        y = np.array([rnd.randrange(m) for _ in range(n)], dtype=np.uint64)
        g = 5
        prod = orc.pointwise("mul", xs[None], y[None], [m])[0]
        assert np.array_equal(orc.automorph_eval(prod, logn, g),
                              orc.pointwise("mul", orc.automorph_eval(xs, logn, g)[None], orc.automorph_eval(y, logn, g)[None], [m])[0])


# ---------------------------------------------------- keys, key switch, HMult, HRot
def _keys(orc, ps, P, rng, sprime_hat, s_hat):
    D = ps.L + ps.K
    a = synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum,))
    e = synth.gaussian_error(rng, (ps.dnum, ps.N))
    return orc.make_switch_key(s_hat, sprime_hat, a, e, P), e


def _setup(orc, ps, seed, hamming=None):
    P = orc.Params.from_set(ps)
    rng = np.random.default_rng(seed)
    s = synth.ternary_hamming(rng, ps.N, hamming) if hamming else synth.ternary_iid(rng, ps.N)
    s_hat = orc.secret_eval(s, P)
    return P, rng, s, s_hat


SHAPES = [(6, 4, 2, 2, 20, 24), (5, 6, 2, 3, 20, 22), (7, 4, 4, 1, 30, 31), (5, 3, 1, 3, 35, 36),
          (5, 5, 3, 2, 20, 24), (5, 7, 3, 3, 20, 22)]   # the last two: dnum does not divide L (digits 3+2 and 3+3+1)


@pytest.mark.parametrize("shape", SHAPES)
def test_switch_key_structure(orc, shape):
    ps = _small_set(*shape)
    P, rng, s, s_hat = _setup(orc, ps, 21)
    s2_hat = orc.pointwise("mul", s_hat, s_hat, ps.primes)
    key, e = _keys(orc, ps, P, rng, s2_hat, s_hat)
    Pp = 1
    for p in ps.p_primes:
        Pp *= p
    for j in range(ps.dnum):
        # key0 + key1*s - gadget_j*s' must be the small error e_j on every limb
        t = orc.pointwise("add", key[j, 0], orc.pointwise("mul", key[j, 1], s_hat, ps.primes), ps.primes)
        gad = np.zeros_like(s2_hat)
        for i in range(j * ps.alpha, min((j + 1) * ps.alpha, ps.L)):
            gad[i] = orc.pointwise("mul", np.full((1, ps.N), Pp % ps.primes[i], dtype=np.uint64), s2_hat[i:i + 1], [ps.primes[i]])[0]
        t = orc.pointwise("sub", t, gad, ps.primes)
        got = orc.centred_small(t, P, ps.L + ps.K)
        assert np.array_equal(got, e[j])


@pytest.mark.parametrize("shape", SHAPES)
def test_keyswitch_decrypt_and_bound(orc, shape):
    ps = _small_set(*shape)
    P, rng, s, s_hat = _setup(orc, ps, 31)
    s2_hat = orc.pointwise("mul", s_hat, s_hat, ps.primes)
    key, _ = _keys(orc, ps, P, rng, s2_hat, s_hat)
    d = synth.uniform_residues(rng, ps.q_primes, ps.N)
    ks = orc.keyswitch(d, key, P)
    E = orc.keyswitch_noise(d, ks, s_hat, s2_hat, P)
    bound = orc.keyswitch_noise_bound(P, int(np.abs(s).sum()))
    assert np.abs(E).max() <= bound
    # the bound is not vacuous: it is far below the modulus
    assert bound < min(ps.q_primes) // 4


@pytest.mark.parametrize("shape", SHAPES)
def test_hmult_relin_decrypts_to_product(orc, shape):
    ps = _small_set(*shape)
    P, rng, s, s_hat = _setup(orc, ps, 41)
    q = ps.q_primes
    s2_hat = orc.pointwise("mul", s_hat, s_hat, ps.primes)
    evk, _ = _keys(orc, ps, P, rng, s2_hat, s_hat)
    ct1 = synth.uniform_residues(rng, q, ps.N, lead=(2,))
    ct2 = synth.uniform_residues(rng, q, ps.N, lead=(2,))
    out = orc.hmult_relin(ct1, ct2, evk, P)
    sq = s_hat[:ps.L]

    def dec(ct):
        return orc.pointwise("add", ct[0], orc.pointwise("mul", ct[1], sq, q), q)

    want = orc.pointwise("mul", dec(ct1), dec(ct2), q)
    E = orc.centred_small(orc.pointwise("sub", dec(out), want, q), P, ps.L)
    assert np.abs(E).max() <= orc.keyswitch_noise_bound(P, int(np.abs(s).sum()))


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("rot", [1, 3, -1])
def test_hrot_decrypts_to_rotated(orc, shape, rot):
    ps = _small_set(*shape)
    P, rng, s, s_hat = _setup(orc, ps, 51)
    q = ps.q_primes
    g = synth.galois_element(rot, ps.logN)
    sg_hat = orc.automorph_limbs(s_hat, P, 0, g, True)
    rk, _ = _keys(orc, ps, P, rng, sg_hat, s_hat)
    ct = synth.uniform_residues(rng, q, ps.N, lead=(2,))
    out = orc.hrot(ct, g, rk, P)
    sq = s_hat[:ps.L]

    def dec(c):
        return orc.pointwise("add", c[0], orc.pointwise("mul", c[1], sq, q), q)

    want = orc.automorph_limbs(dec(ct), P, 0, g, True)
    E = orc.centred_small(orc.pointwise("sub", dec(out), want, q), P, ps.L)
    assert np.abs(E).max() <= orc.keyswitch_noise_bound(P, int(np.abs(s).sum()))


@pytest.mark.parametrize("shape", SHAPES[:2])
def test_hoisted_mac_per_rotation_and_linearity(orc, shape):
    ps = _small_set(*shape)
    P, rng, s, s_hat = _setup(orc, ps, 61)
    q = ps.q_primes
    rots = [1, 2, -1, 5]
    gs = [synth.galois_element(r, ps.logN) for r in rots]
    rks = []
    for g in gs:
        sg_hat = orc.automorph_limbs(s_hat, P, 0, g, True)
        rks.append(_keys(orc, ps, P, rng, sg_hat, s_hat)[0])
    ct = synth.uniform_residues(rng, q, ps.N, lead=(2,))
    pt = synth.uniform_residues(rng, q, ps.N, lead=(len(rots),))
    out, per = orc.hrot_hoisted_mac(ct, gs, rks, pt, P, want_per_rotation=True)
    sq = s_hat[:ps.L]

    def dec(c):
        return orc.pointwise("add", c[0], orc.pointwise("mul", c[1], sq, q), q)

    bound = orc.keyswitch_noise_bound(P, int(np.abs(s).sum()))
    acc = np.zeros((2, ps.L, ps.N), dtype=np.uint64)
    differs = False
    for r, g in enumerate(gs):
        want = orc.automorph_limbs(dec(ct), P, 0, g, True)
        E = orc.centred_small(orc.pointwise("sub", dec(per[r]), want, q), P, ps.L)
        assert np.abs(E).max() <= bound
        for t in range(2):
            acc[t] = orc.pointwise("add", acc[t], orc.pointwise("mul", pt[r], per[r, t], q), q)
        # unit plaintext (all ones in evaluation form) on rotation r alone reproduces R_r
        unit = np.zeros_like(pt)
        unit[r] = 1
        assert np.array_equal(orc.hrot_hoisted_mac(ct, gs, rks, unit, P), per[r])
        differs |= not np.array_equal(orc.hrot(ct, g, rks[r], P), per[r])
    assert np.array_equal(acc, out)
    assert differs  # hoisted and un-hoisted rotations agree only up to noise, not bit for bit


def test_config0_exact_shape_hmult(orc):
    """workload 0: N=2^12, 3 q-limbs above 2^35, one special prime above 2^36, dnum=3."""
    ps = synth.CFG0
    P, rng, s, s_hat = _setup(orc, ps, 0)
    q = ps.q_primes
    s2_hat = orc.pointwise("mul", s_hat, s_hat, ps.primes)
    evk, _ = _keys(orc, ps, P, rng, s2_hat, s_hat)
    ct1 = synth.uniform_residues(rng, q, ps.N, lead=(2,))
    ct2 = synth.uniform_residues(rng, q, ps.N, lead=(2,))
    out = orc.hmult_relin(ct1, ct2, evk, P)
    sq = s_hat[:ps.L]

    def dec(ct):
        return orc.pointwise("add", ct[0], orc.pointwise("mul", ct[1], sq, q), q)

    E = orc.centred_small(orc.pointwise("sub", dec(out), orc.pointwise("mul", dec(ct1), dec(ct2), q), q), P, ps.L)
    bound = orc.keyswitch_noise_bound(P, int(np.abs(s).sum()))
    assert bound <= 116736 + 4097 + 1
    assert 0 < np.abs(E).max() <= bound


# ------------------------------------------------------ levels below L and rescale
def _negacyclic_int(a, b):
    """Integer negacyclic product (no modulus) of two integer lists."""
    n = len(a)
    out = [0] * n
    for i, ai in enumerate(a):
        if ai == 0:
            continue
        for j, bj in enumerate(b):
            k = i + j
            if k < n:
                out[k] += ai * bj
            else:
                out[k - n] -= ai * bj
    return out


def _coeff(orc, x, P, n_limbs):
    return orc.ntt_batch(np.ascontiguousarray(x[:n_limbs]), P, 0, inverse=True)


@pytest.mark.parametrize("ell", [5, 4, 2])
def test_rescale_vs_bigint_floor_division(orc, ell):
    ps = _small_set(4, 5, 1, 5, 30, 31)
    P = orc.Params.from_set(ps)
    q = list(ps.q_primes[:ell])
    rng = np.random.default_rng(71 + ell)
    c = synth.uniform_residues(rng, q, ps.N)
    Qe = 1
    for m in q:
        Qe *= m
    big = (123456789123456789 * 987654321987 % (Qe // q[-1])) * q[-1]       # coefficient 0: exact multiple
    small = q[-1] - 1                                                         # coefficient 1: below the divisor
    for i, m in enumerate(q):
        c[i, 0], c[i, 1] = big % m, small % m
    x = orc.ntt_batch(c, P, 0)
    out = orc.rescale(x, P)
    assert out.shape == (ell - 1, ps.N)
    oc = _coeff(orc, out, P, ell - 1)
    for n in range(ps.N):
        X, _ = crt([c[i, n] for i in range(ell)], q)
        want = (X - X % q[-1]) // q[-1]
        assert [int(oc[i, n]) for i in range(ell - 1)] == [want % m for m in q[:-1]]
    assert all(int(oc[i, 0]) == (big // q[-1]) % q[i] for i in range(ell - 1))
    assert all(int(oc[i, 1]) == 0 for i in range(ell - 1))


def test_rescale_decryption_identity(orc):
    """q_last * Dec(rescale(ct)) - Dec(ct) = -([b]_q + [a]_q * s) exactly (mod Q_ell), [.]_q in [0, q_last)."""
    ps = _small_set(5, 4, 2, 2, 24, 26)
    P, rng, s, s_hat = _setup(orc, ps, 73)
    for ell in (4, 3):
        q = list(ps.q_primes[:ell])
        ct = synth.uniform_residues(rng, q, ps.N, lead=(2,))
        out = orc.rescale(ct, P)
        assert out.shape == (2, ell - 1, ps.N)

        def dec(c, n_l):
            qq = q[:n_l]
            return orc.pointwise("add", c[0], orc.pointwise("mul", c[1], s_hat[:n_l], qq), qq)

        m_c = _coeff(orc, dec(ct, ell), P, ell)
        m2_c = _coeff(orc, dec(out, ell - 1), P, ell - 1)
        r0 = orc.intt(ct[0, ell - 1], ps.logN, q[-1], P.psi[ell - 1]).tolist()
        r1 = orc.intt(ct[1, ell - 1], ps.logN, q[-1], P.psi[ell - 1]).tolist()
        r1s = _negacyclic_int([int(v) for v in r1], [int(v) for v in s])
        Qe = 1
        for m in q:
            Qe *= m
        worst = 0
        for n in range(ps.N):
            M, _ = crt([m_c[i, n] for i in range(ell)], q)
            M2, _ = crt([m2_c[i, n] for i in range(ell - 1)], q[:-1])
            E = (q[-1] * M2 - M) % Qe
            E = E - Qe if E > Qe // 2 else E
            assert E == -(int(r0[n]) + r1s[n])
            worst = max(worst, abs(E))
        assert worst <= q[-1] * (1 + int(np.abs(s).sum())) < Qe // 4


LEVEL_SHAPES = [(5, 6, 2, 3, 20, 22), (5, 6, 3, 2, 20, 24), (4, 8, 2, 4, 49, 59)]


@pytest.mark.parametrize("shape", LEVEL_SHAPES)
def test_modup_level_vs_bigint_crt(orc, shape):
    ps = _small_set(*shape)
    P = orc.Params.from_set(ps)
    rng = np.random.default_rng(75)
    a = ps.alpha
    for ell in range(1, ps.L + 1):
        x = synth.uniform_residues(rng, ps.q_primes[:ell], ps.N)
        out = orc.modup_level(x, P)
        beta = -(-ell // a)
        basis = list(ps.q_primes[:ell]) + list(ps.p_primes)
        assert out.shape == (beta, ell + ps.K, ps.N)
        for j in range(beta):
            lo, hi = j * a, min((j + 1) * a, ell)
            digit = basis[lo:hi]
            for n in range(0, ps.N, 3):
                xi, Qj = crt([x[i, n] for i in range(lo, hi)], digit)
                us = set()
                for t, b in enumerate(basis):
                    if lo <= t < hi:
                        assert out[j, t, n] == x[t, n]
                        continue
                    us.add((int(out[j, t, n]) - xi) * pow(Qj, -1, b) % b)
                assert len(us) == 1 and 0 <= us.pop() < hi - lo
        if ell == ps.L:
            assert np.array_equal(out, orc.modup(x, P))


@pytest.mark.parametrize("shape", LEVEL_SHAPES[:2] + [(6, 4, 4, 1, 30, 31)])
def test_keyswitch_level_decrypt_and_bound(orc, shape):
    ps = _small_set(*shape)
    P, rng, s, s_hat = _setup(orc, ps, 77)
    s2_hat = orc.pointwise("mul", s_hat, s_hat, ps.primes)
    key, _ = _keys(orc, ps, P, rng, s2_hat, s_hat)
    for ell in range(1, ps.L + 1):
        d = synth.uniform_residues(rng, ps.q_primes[:ell], ps.N)
        ks = orc.keyswitch_level(d, key, P)
        assert ks.shape == (2, ell, ps.N)
        E = orc.keyswitch_noise(d, ks, s_hat, s2_hat, P, level=ell)
        bound = orc.keyswitch_noise_bound(P, int(np.abs(s).sum()), level=ell)
        assert np.abs(E).max() <= bound
        assert ell == 1 or bound < min(ps.q_primes) // 4
        if ell == ps.L:
            assert np.array_equal(ks, orc.keyswitch(d, key, P))     # the full level is the special case


@pytest.mark.parametrize("shape", LEVEL_SHAPES[:2])
def test_hmult_hrot_level_decrypt(orc, shape):
    ps = _small_set(*shape)
    P, rng, s, s_hat = _setup(orc, ps, 79)
    s2_hat = orc.pointwise("mul", s_hat, s_hat, ps.primes)
    evk, _ = _keys(orc, ps, P, rng, s2_hat, s_hat)
    g = synth.galois_element(3, ps.logN)
    sg_hat = orc.automorph_limbs(s_hat, P, 0, g, True)
    rk, _ = _keys(orc, ps, P, rng, sg_hat, s_hat)
    for ell in (ps.L, ps.L - 1, ps.alpha + 1, 1):
        q = list(ps.q_primes[:ell])
        sq = s_hat[:ell]

        def dec(c):
            return orc.pointwise("add", c[0], orc.pointwise("mul", c[1], sq, q), q)

        bound = orc.keyswitch_noise_bound(P, int(np.abs(s).sum()), level=ell)
        ct1 = synth.uniform_residues(rng, q, ps.N, lead=(2,))
        ct2 = synth.uniform_residues(rng, q, ps.N, lead=(2,))
        out = orc.hmult_relin_level(ct1, ct2, evk, P)
        E = orc.centred_small(orc.pointwise("sub", dec(out), orc.pointwise("mul", dec(ct1), dec(ct2), q), q), P, ell)
        assert np.abs(E).max() <= bound
        rot = orc.hrot_level(ct1, g, rk, P)
        E = orc.centred_small(orc.pointwise("sub", dec(rot), orc.automorph_limbs(dec(ct1), P, 0, g, True), q), P, ell)
        assert np.abs(E).max() <= bound
        if ell == ps.L:
            assert np.array_equal(out, orc.hmult_relin(ct1, ct2, evk, P))
            assert np.array_equal(rot, orc.hrot(ct1, g, rk, P))


def test_hoisted_mac_level(orc):
    ps = _small_set(5, 6, 2, 3, 20, 22)
    P, rng, s, s_hat = _setup(orc, ps, 81)
    rots = [1, -2, 4]
    gs = [synth.galois_element(r, ps.logN) for r in rots]
    rks = [_keys(orc, ps, P, rng, orc.automorph_limbs(s_hat, P, 0, g, True), s_hat)[0] for g in gs]
    for ell in (ps.L, 5, 3):
        q = list(ps.q_primes[:ell])
        sq = s_hat[:ell]

        def dec(c):
            return orc.pointwise("add", c[0], orc.pointwise("mul", c[1], sq, q), q)

        ct = synth.uniform_residues(rng, q, ps.N, lead=(2,))
        pt = synth.uniform_residues(rng, q, ps.N, lead=(len(rots),))
        out = orc.hrot_hoisted_mac_level(ct, gs, rks, pt, P)
        if ell == ps.L:
            assert np.array_equal(out, orc.hrot_hoisted_mac(ct, gs, rks, pt, P))
        bound = orc.keyswitch_noise_bound(P, int(np.abs(s).sum()), level=ell)
        acc = np.zeros_like(out)
        for r, g in enumerate(gs):
            unit = np.ones((1, ell, ps.N), dtype=np.uint64)            # NTT(1): rotation r alone, unscaled
            one = orc.hrot_hoisted_mac_level(ct, [g], [rks[r]], unit, P)
            E = orc.centred_small(orc.pointwise("sub", dec(one), orc.automorph_limbs(dec(ct), P, 0, g, True), q), P, ell)
            assert np.abs(E).max() <= bound
            for t in range(2):
                acc[t] = orc.pointwise("add", acc[t], orc.pointwise("mul", pt[r], one[t], q), q)
        assert np.array_equal(acc, out)                               # linear in the per-rotation results


# ------------------------------------------------------------- double hoisting
def _small_plaintexts(orc, rng, P, n_rot, ell, amp=4):
    """Plaintext polynomials with coefficients in [-amp, amp], reduced modulo every prime of the level's
    extended basis and transformed: [n_rot][ell+K][N], plus their l1 norms."""
    basis = list(P.primes[:ell]) + list(P.primes[P.L:])
    psis = list(P.psi[:ell]) + list(P.psi[P.L:])
    coeffs = rng.integers(-amp, amp + 1, size=(n_rot, P.N))
    out = np.empty((n_rot, len(basis), P.N), dtype=np.uint64)
    for r in range(n_rot):
        lifted = orc.lift_signed(coeffs[r], basis)
        for i, (m, w) in enumerate(zip(basis, psis)):
            out[r, i] = orc.ntt(lifted[i], P.logN, m, w)
    return out, [int(np.abs(c).sum()) for c in coeffs]


@pytest.mark.parametrize("shape", LEVEL_SHAPES[:2] + [(6, 4, 4, 1, 30, 31)])
def test_double_hoisted_mac_decrypts_and_reduces_to_single_rotation(orc, shape):
    ps = _small_set(*shape)
    P, rng, s, s_hat = _setup(orc, ps, 91)
    rots = [1, -2, 4, 7]
    gs = [synth.galois_element(r, ps.logN) for r in rots]
    rks = [_keys(orc, ps, P, rng, orc.automorph_limbs(s_hat, P, 0, g, True), s_hat)[0] for g in gs]
    h = int(np.abs(s).sum())
    for ell in sorted({ps.L, ps.L - 1, min(ps.alpha + 1, ps.L), 1}):
        q = list(ps.q_primes[:ell])
        sq = s_hat[:ell]

        def dec(c):
            return orc.pointwise("add", c[0], orc.pointwise("mul", c[1], sq, q), q)

        ct = synth.uniform_residues(rng, q, ps.N, lead=(2,))
        pt, l1 = _small_plaintexts(orc, rng, P, len(rots), ell)
        out = orc.hrot_dh_mac_level(ct, gs, rks, pt, P)
        want = np.zeros((ell, ps.N), dtype=np.uint64)
        for r, g in enumerate(gs):
            want = orc.pointwise("add", want, orc.pointwise("mul", pt[r, :ell], orc.automorph_limbs(dec(ct), P, 0, g, True), q), q)
        E = orc.centred_small(orc.pointwise("sub", dec(out), want, q), P, ell)
        bound = orc.dh_mac_noise_bound(P, h, sum(l1), level=ell)
        assert np.abs(E).max() <= bound
        assert ell == 1 or bound < min(q) // 4
        # one rotation with the unit plaintext is exactly the singly hoisted rotation
        unit = np.ones((1, ell + ps.K, ps.N), dtype=np.uint64)
        for r in (0, 3):
            one = orc.hrot_dh_mac_level(ct, [gs[r]], [rks[r]], unit, P)
            assert np.array_equal(one, orc.hrot_hoisted_mac_level(ct, [gs[r]], [rks[r]], unit[:, :ell], P))
        # ... but the sum over rotations is not the sum of singly hoisted terms bit for bit
        single = orc.hrot_hoisted_mac_level(ct, gs, rks, np.ascontiguousarray(pt[:, :ell]), P)
        assert ell == 1 or not np.array_equal(single, out)
        Es = orc.centred_small(orc.pointwise("sub", dec(single), dec(out), q), P, ell)
        assert np.abs(Es).max() <= bound + sum(l1) * (ps.K * (1 + h) + 1) + sum(l1)


# ------------------------------------------------ ModDown merged with the rescale
@pytest.mark.parametrize("shape", [(5, 4, 2, 2, 20, 24), (4, 6, 3, 2, 20, 22), (4, 3, 1, 3, 35, 36), (4, 8, 2, 4, 49, 59)])
def test_moddown_merged_vs_bigint(orc, shape):
    ps = _small_set(*shape)
    P = orc.Params.from_set(ps)
    rng = np.random.default_rng(93)
    for ell in sorted({ps.L, ps.L - 1, 2}):
        basis = list(ps.q_primes[:ell]) + list(ps.p_primes)
        S = basis[ell - 1:]
        PS = 1
        for m in S:
            PS *= m
        Qt = 1
        for m in basis[:ell - 1]:
            Qt *= m
        x = synth.uniform_residues(rng, basis, ps.N)
        big = (rng.integers(0, 2**62, dtype=np.uint64).item() * 987654321987654321 % Qt) * PS   # exact multiple
        for t, m in enumerate(basis):
            x[t, 0] = big % m
        out = orc.moddown_merged(x, P)
        assert out.shape == (ell - 1, ps.N)
        for n in range(ps.N):
            c, _ = crt([x[t, n] for t in range(len(basis))], basis)
            us = {(c // PS - int(out[i, n])) % q for i, q in enumerate(basis[:ell - 1])}
            assert len(us) == 1
            u = us.pop()
            assert 0 <= u <= ps.K                                                     # K+1 sources
            if n == 0:
                assert u == 0 and all(int(out[i, 0]) == (big // PS) % q for i, q in enumerate(basis[:ell - 1]))


@pytest.mark.parametrize("shape", LEVEL_SHAPES[:2] + [(6, 4, 4, 1, 30, 31)])
def test_hmult_relin_rescale_merged_stays_next_to_the_two_step_result(orc, shape):
    ps = _small_set(*shape)
    P, rng, s, s_hat = _setup(orc, ps, 95)
    s2_hat = orc.pointwise("mul", s_hat, s_hat, ps.primes)
    evk, _ = _keys(orc, ps, P, rng, s2_hat, s_hat)
    seen_different = False
    for ell in range(ps.L, 1, -1):
        q = list(ps.q_primes[:ell])
        ct1 = synth.uniform_residues(rng, q, ps.N, lead=(2,))
        ct2 = synth.uniform_residues(rng, q, ps.N, lead=(2,))
        merged = orc.hmult_relin_rescale_level(ct1, ct2, evk, P)
        two_step = orc.rescale(orc.hmult_relin_level(ct1, ct2, evk, P), P)
        assert merged.shape == two_step.shape == (2, ell - 1, ps.N)
        for t in range(2):
            diff = orc.centred_small(orc.pointwise("sub", merged[t], two_step[t], q[:-1]), P, ell - 1)
            # merged = floor(X/(P q)) - u2, u2 in [0, K]; two-step = that floor or one less: diff in [-K, 1]
            assert -ps.K <= diff.min() and diff.max() <= 1
        seen_different |= not np.array_equal(merged, two_step)
    assert seen_different


@pytest.mark.parametrize("shape", LEVEL_SHAPES[:2])
def test_double_hoisted_mac_rescale_merged_stays_next_to_the_two_step_result(orc, shape):
    ps = _small_set(*shape)
    P, rng, s, s_hat = _setup(orc, ps, 97)
    gs = [synth.galois_element(r, ps.logN) for r in (1, -2, 4)]
    rks = [_keys(orc, ps, P, rng, orc.automorph_limbs(s_hat, P, 0, g, True), s_hat)[0] for g in gs]
    seen_different = False
    for ell in range(ps.L, 1, -1):
        q = list(ps.q_primes[:ell])
        ct = synth.uniform_residues(rng, q, ps.N, lead=(2,))
        pt = synth.uniform_residues(rng, q + list(ps.p_primes), ps.N, lead=(len(gs),))
        merged = orc.hrot_dh_mac_rescale_level(ct, gs, rks, pt, P)
        two_step = orc.rescale(orc.hrot_dh_mac_level(ct, gs, rks, pt, P), P)
        for t in range(2):
            diff = orc.centred_small(orc.pointwise("sub", merged[t], two_step[t], q[:-1]), P, ell - 1)
            assert -ps.K <= diff.min() and diff.max() <= 1
        seen_different |= not np.array_equal(merged, two_step)
    assert seen_different


# ------------------------------------------------- baby-step giant-step transform
def test_bsgs_linear_transform_decrypts_to_the_sum_of_rotated_products(orc):
    """Dec(out) = sum_g sum_b sigma_G(pt[g][b]) * sigma_{G*g_b}(m) up to the noise of n2 double-hoisted sums
    (each rotated once more) and n2 key switches."""
    ps = _small_set(6, 6, 2, 3, 20, 22)
    P, rng, s, s_hat = _setup(orc, ps, 101)
    h = int(np.abs(s).sum())
    baby = [synth.galois_element(r, ps.logN) for r in (0, 1, 2)]
    giant = [synth.galois_element(r, ps.logN) for r in (0, 3)]
    baby_rks = [_keys(orc, ps, P, rng, orc.automorph_limbs(s_hat, P, 0, g, True), s_hat)[0] for g in baby]
    giant_rks = [_keys(orc, ps, P, rng, orc.automorph_limbs(s_hat, P, 0, g, True), s_hat)[0] for g in giant]
    for ell in (ps.L, 3):
        q = list(ps.q_primes[:ell])
        sq = s_hat[:ell]

        def dec(c):
            return orc.pointwise("add", c[0], orc.pointwise("mul", c[1], sq, q), q)

        ct = synth.uniform_residues(rng, q, ps.N, lead=(2,))
        pts, l1s = [], []
        for g in giant:
            ptg, l1 = _small_plaintexts(orc, rng, P, len(baby), ell, amp=2)
            pts.append(ptg)
            l1s.append(sum(l1))
        pt = np.stack(pts)
        out = orc.lintrans_bsgs_level(ct, baby, baby_rks, giant, giant_rks, pt, P)
        want = np.zeros((ell, ps.N), dtype=np.uint64)
        m = dec(ct)
        for gi, G in enumerate(giant):
            for bi, gb in enumerate(baby):
                term = orc.pointwise("mul", pt[gi, bi, :ell], orc.automorph_limbs(m, P, 0, gb, True), q)
                want = orc.pointwise("add", want, orc.automorph_limbs(term, P, 0, G, True), q)
        E = orc.centred_small(orc.pointwise("sub", dec(out), want, q), P, ell)
        bound = sum(orc.dh_mac_noise_bound(P, h, l1, level=ell) for l1 in l1s) \
            + len(giant) * orc.keyswitch_noise_bound(P, h, level=ell)
        assert 0 < np.abs(E).max() <= bound < min(q) // 4
        # a single giant step with the identity-free structure reduces to its parts
        one = orc.lintrans_bsgs_level(ct, baby, baby_rks, giant[1:], giant_rks[1:], pt[1:], P)
        inner = orc.hrot_dh_mac_level(ct, baby, baby_rks, pt[1], P)
        assert np.array_equal(one, orc.hrot_level(inner, giant[1], giant_rks[1], P))


def test_level_functions_at_the_full_level_equal_the_full_level_functions(orc):
    """The level functions (digits of ceil(L/dnum) limbs, last digit possibly shorter) are the definition used when
    dnum does not divide L; with equal digits they must reproduce the full-level functions word for word."""
    ps = _small_set(5, 6, 2, 3, 20, 22)
    P = orc.Params.from_set(ps)
    rng = np.random.default_rng(91)
    key = synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2))
    ct1 = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(2,))
    ct2 = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(2,))
    g = synth.galois_element(3, ps.logN)
    assert np.array_equal(orc.keyswitch_level(ct1[0], key, P), orc.keyswitch(ct1[0], key, P))
    assert np.array_equal(orc.hmult_relin_level(ct1, ct2, key, P), orc.hmult_relin(ct1, ct2, key, P))
    assert np.array_equal(orc.hrot_level(ct1, g, key, P), orc.hrot(ct1, g, key, P))
    x = synth.uniform_residues(rng, ps.q_primes, ps.N)
    assert np.array_equal(orc.modup_level(x, P), orc.modup(x, P))
    gs = [g, synth.galois_element(-1, ps.logN)]
    pt = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(2,))
    assert np.array_equal(orc.hrot_hoisted_mac_level(ct1, gs, [key, key], pt, P), orc.hrot_hoisted_mac(ct1, gs, [key, key], pt, P))


# --------------------------------------------------- encoded diagonals: matrix-vector products on the slots
def _centred(limb, q):
    v = limb.astype(np.int64)
    return np.where(limb > np.uint64(q // 2), v - q, v)


def test_canonical_embedding_pins(orc):
    """encode/decode against what fixes them: the evaluation points are roots of X^N + 1, a constant slot vector is
    a constant polynomial, decode inverts encode within the rounding bound, the embedding is multiplicative
    (big-integer negacyclic product), and the automorphism with Galois element 5^r rotates the slots by r
    (2N - 1 conjugates them) -- the convention every rotation key and diagonal below relies on."""
    logN, scale = 5, float(1 << 30)
    n = 1 << logN
    zeta = orc.slot_roots(logN)
    assert np.abs(zeta ** n + 1).max() < 1e-12 and len(set(np.round(zeta, 9))) == n // 2
    assert np.abs(np.abs(np.subtract.outer(zeta, np.conj(zeta)))).min() > 1e-3          # one of each conjugate pair
    m = orc.encode(np.full(n // 2, 0.75), scale, logN)
    assert m[0] == int(0.75 * scale) and not m[1:].any()
    rng = np.random.default_rng(11)
    z = rng.uniform(-1, 1, n // 2) + 1j * rng.uniform(-1, 1, n // 2)
    w = rng.uniform(-1, 1, n // 2) + 1j * rng.uniform(-1, 1, n // 2)
    mz, mw = orc.encode(z, scale, logN), orc.encode(w, scale, logN)
    # rounding moves every coefficient by at most 1/2, a slot by at most N/2
    assert np.abs(orc.decode(mz, scale, logN) - z).max() <= n / 2 / scale
    prod = negacyclic_schoolbook([int(v) for v in mz], [int(v) for v in mw], 1 << 200)
    prod = [v - (1 << 200) if v >> 199 else v for v in prod]
    got = orc.decode(np.array(prod, dtype=np.float64), scale * scale, logN)
    assert np.abs(got - z * w).max() <= 4 * n / scale
    q = synth.primes_above(1 << 49, 2 * n, 1)[0]
    lifted = orc.lift_signed(mz, [q])[0]
    for r in (1, 3, -1, n // 4):
        rot = _centred(orc.automorph_coeff(lifted, logN, q, synth.galois_element(r, logN)), q)
        assert np.abs(orc.decode(rot, scale, logN) - np.roll(z, -r)).max() <= n / scale, r
    conj = _centred(orc.automorph_coeff(lifted, logN, q, 2 * n - 1), q)
    assert np.abs(orc.decode(conj, scale, logN) - np.conj(z)).max() <= n / scale
    # diagonals: M z = sum_d diag_d * rot_d(z)
    M = rng.uniform(-1, 1, (n // 2, n // 2))
    acc = sum(orc.matrix_diagonal(M, d) * np.roll(z, -d) for d in range(n // 2))
    assert np.abs(acc - M @ z).max() < 1e-12


def test_bsgs_with_encoded_diagonals_is_the_matrix_vector_product(orc):
    """A dense 32 x 32 complex matrix on the 32 slots of N = 64, cut into 8 x 4 diagonals and encoded: the baby-step
    giant-step call on an encryption of z decrypts and decodes to M z within the stated error (rounding of the two
    encodings, the fresh encryption error, and the key-switch noise bound of the call)."""
    ps = _small_set(6, 4, 2, 2, 49, 59)
    P, rng, s, s_hat = _setup(orc, ps, 77)
    h = int(np.abs(s).sum())
    N, n = ps.N, ps.N // 2
    n1, n2 = 8, 4
    scale = scale_pt = float(1 << 25)
    M = (rng.uniform(-1, 1, (n, n)) + 1j * rng.uniform(-1, 1, (n, n))) / np.sqrt(2)      # entries of modulus <= 1
    z = (rng.uniform(-1, 1, n) + 1j * rng.uniform(-1, 1, n)) / np.sqrt(2)
    baby = [synth.galois_element(b, ps.logN) for b in range(n1)]
    giant = [synth.galois_element(g * n1, ps.logN) for g in range(n2)]
    baby_rks = [_keys(orc, ps, P, rng, orc.automorph_limbs(s_hat, P, 0, g, True), s_hat)[0] for g in baby]
    giant_rks = [_keys(orc, ps, P, rng, orc.automorph_limbs(s_hat, P, 0, g, True), s_hat)[0] for g in giant]
    for ell in (ps.L, 3):
        q = list(ps.q_primes[:ell])
        sq = s_hat[:ell]
        # fresh encryption of encode(z): b = -a*s + m + e
        m_hat = orc.encode_limbs(z, scale, P, q, P.psi[:ell])
        a = synth.uniform_residues(rng, q, N)
        e = synth.gaussian_error(rng, (N,))
        e_hat = orc.ntt_batch(orc.lift_signed(e, q), P, 0)
        b = orc.pointwise("add", orc.pointwise("sub", m_hat, orc.pointwise("mul", a, sq, q), q), e_hat, q)
        ct = np.stack([b, a])
        pt = orc.bsgs_diagonal_plaintexts(M, n1, n2, scale_pt, P, ell)
        out = orc.lintrans_bsgs_level(ct, baby, baby_rks, giant, giant_rks, pt, P)
        dec = orc.pointwise("add", out[0], orc.pointwise("mul", out[1], sq, q), q)
        coeffs = orc.crt_centred(dec, P, ell)                    # about 2^55: small against Q, not against one limb
        assert max(abs(v) for v in coeffs) < (1 << 60)
        got = orc.decode(np.array(coeffs, dtype=np.float64), scale * scale_pt, ps.logN)
        # l1 norms of the encoded diagonals, per giant step, for the noise bound of the double-hoisted sums
        basis = q + list(ps.p_primes)
        l1 = []
        for g in range(n2):
            tot = 0
            for bb in range(n1):
                tot += int(np.abs(orc.centred_small(pt[g, bb], P, ell)).sum())
            l1.append(tot)
        noise = sum(orc.dh_mac_noise_bound(P, h, t, level=ell) for t in l1) + n2 * orc.keyswitch_noise_bound(P, h, level=ell)
        # slot-domain error: a coefficient error c moves a slot by at most N*c; every slot sums n products
        tol = n * (N / 2 + 19 * N) / scale + n * (N / 2) / scale_pt + N * noise / (scale * scale_pt)
        err = np.abs(got - M @ z).max()
        assert err <= tol < 0.01, (ell, err, tol)
        assert err > 0
        del basis

def test_eval_automorphism_maps_256_slot_rows_onto_rows(orc):
    """In evaluation (bit-reversed) order sigma_g sends every aligned block of 256 slots to one aligned source
    block: the block index is the bit-reversed low part of the exponent index, and multiplying the odd exponent by
    an odd g keeps low parts among themselves.  The kernels rely on it when they fetch a rotation's source row
    whole and permute it on chip; here it is read off the oracle's own permutation (independent code), for
    rotations, their inverses and the conjugation, at every ring degree the library accepts."""
    for logn in (12, 13, 16):
        n = 1 << logn
        ident = np.arange(n, dtype=np.uint64)
        gs = [synth.galois_element(r, logn) for r in (1, 2, 3, 7, 64, 1000, -1, -5)] + [2 * n - 1, 3, 2 * n - 3]
        for g in gs:
            assert g % 2 == 1
            src = orc.automorph_eval(ident, logn, g)          # out[j] = in[src[j]]
            assert sorted(src.tolist()) == list(range(n))     # a permutation
            rows = (src >> np.uint64(8)).reshape(n // 256, 256)
            assert (rows == rows[:, :1]).all(), (logn, g)     # one source row per destination row
            assert sorted(rows[:, 0].tolist()) == list(range(n // 256))
