"""Parity on prime chains that mix sizes and arithmetic classes (needs an MI355X).

The benchmark chains are uniform (50-bit q-limbs, 60-bit special limbs).  Here neighbouring limbs
alternate between the FP64 and the integer arithmetic, some conversion targets are too small for
their sources to be converted on the FP64 pipe (the library then converts them with integers), one
prime lies below 2^28, and two pairs straddle the bound between the two arithmetics.  Everything is
compared bit for bit with the oracle; nothing here depends on noise being small.
"""
import numpy as np
import pytest

from paper_2310_16530_amd import synth

from test_gpu_parity import dev, gpu_ctx, host, orc_params

pytestmark = pytest.mark.gpu

FP_LIMIT = 3 << 48
CHAINS = {
    "alternating": (12, [36, 50, 30, 27, 55, 49], [59, 40], 3),
    "big_small": (13, [60, 28, 49, 49], [36, 36, 60], 2),
    "class_boundary": (12, [FP_LIMIT - (1 << 20), FP_LIMIT - (1 << 20), FP_LIMIT, FP_LIMIT], [FP_LIMIT - (1 << 22), 59], 2),
    "small_special": (14, [50, 50, 50], [30, 31, 32], 1),
    # digits of 10 limbs (more than one accumulation round in the conversions), both classes among sources and targets
    "wide_digits": (12, [50, 36, 55, 49, 60, 50, 30, 49, 50, 58] * 2, [59, 40, 60, 50, 59, 36, 60, 49, 59, 45], 2),
}


def _say(*a):
    print(*a, flush=True)


@pytest.mark.parametrize("name", sorted(CHAINS))
def test_every_entry_point_on_a_mixed_chain(orc, name):
    logN, qf, pf, dnum = CHAINS[name]
    ps = synth.mixed_params(logN, qf, pf, dnum, name)
    if name == "class_boundary":
        assert [p < FP_LIMIT for p in ps.primes] == [True, True, False, False, True, False]
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = np.random.default_rng(len(name) * 1000 + logN)
    L, K, N, D = ps.L, ps.K, ps.N, ps.L + ps.K
    _say(name, "transforms")
    x = synth.uniform_residues(rng, ps.primes, N, lead=(2,))
    for i, p in enumerate(ps.primes):
        x[1, i, :5] = p - 1
    assert np.array_equal(host(ctx.ntt(dev(x))), orc.ntt_batch(x, P, 0))
    assert np.array_equal(host(ctx.intt(dev(x))), orc.ntt_batch(x, P, 0, inverse=True))
    _say(name, "conversions")
    c = synth.uniform_residues(rng, ps.q_primes, N, lead=(2,))
    up = host(ctx.modup(dev(c)))
    for b in range(2):
        assert np.array_equal(up[b], orc.modup(c[b], P))
    assert np.array_equal(host(ctx.moddown(dev(x)))[0], orc.moddown(x[0], P))
    key = synth.uniform_residues(rng, ps.primes, N, lead=(ps.dnum, 2))
    d_key = dev(key)
    g = synth.galois_element(7, logN)
    gs = [synth.galois_element(r, logN) for r in (1, -1, 5)]
    rks = [synth.uniform_residues(rng, ps.primes, N, lead=(ps.dnum, 2)) for _ in gs]
    d_rks = [dev(k) for k in rks]
    for ell in range(L, 0, -1):
        _say(name, "level", ell)
        q = ps.q_primes[:ell]
        ct1 = synth.uniform_residues(rng, q, N, lead=(2, 2))
        ct2 = synth.uniform_residues(rng, q, N, lead=(2, 2))
        ks = host(ctx.keyswitch_at(ell, dev(ct1[:, 0]), d_key))
        hm = host(ctx.hmult_relin_at(ell, dev(ct1), dev(ct2), d_key))
        hr = host(ctx.hrot_at(ell, dev(ct1), g, d_key))
        for b in range(2):
            assert np.array_equal(ks[b], orc.keyswitch_level(ct1[b, 0], key, P)), (ell, b)
            assert np.array_equal(hm[b], orc.hmult_relin_level(ct1[b], ct2[b], key, P)), (ell, b)
            assert np.array_equal(hr[b], orc.hrot_level(ct1[b], g, key, P)), (ell, b)
        basis = list(q) + list(ps.p_primes)
        pt = synth.uniform_residues(rng, basis, N, lead=(len(gs),))
        ho = host(ctx.hrot_hoisted_mac_at(ell, dev(ct1[0]), gs, d_rks, dev(pt[:, :ell])))
        assert np.array_equal(ho, orc.hrot_hoisted_mac_level(ct1[0], gs, rks, np.ascontiguousarray(pt[:, :ell]), P)), ell
        dh = host(ctx.hrot_dh_mac(dev(ct1[0]), gs, d_rks, dev(pt), level=ell))
        assert np.array_equal(dh, orc.hrot_dh_mac_level(ct1[0], gs, rks, pt, P)), ell
        if ell >= 2:
            assert np.array_equal(host(ctx.rescale(ell, dev(ct1))), orc.rescale(ct1, P)), ell


@pytest.mark.parametrize("shape,levels", [((12, 56, 8, 7), (56, 51, 9)), ((12, 60, 15, 4), (60, 46, 16)),
                                          ((12, 112, 16, 7), (112, 33))])
def test_long_chains(orc, shape, levels):
    """Long chains at N = 2^12: 64 primes in digits of 8, the paper's upper end L = 60 in four digits of 15, and
    L + K = 128 primes (the limit) with digits and a special basis of 16 limbs (both limits)."""
    ps = synth.small_params(*shape)
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = np.random.default_rng(64)
    key = synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2))
    d_key = dev(key)
    g = synth.galois_element(3, ps.logN)
    for ell in levels:
        _say("long chain", shape, "level", ell)
        q = ps.q_primes[:ell]
        ct1 = synth.uniform_residues(rng, q, ps.N, lead=(2, 2))
        ct2 = synth.uniform_residues(rng, q, ps.N, lead=(2, 2))
        hm = host(ctx.hmult_relin_at(ell, dev(ct1), dev(ct2), d_key))
        hr = host(ctx.hrot_at(ell, dev(ct1), g, d_key))
        for b in range(2):
            assert np.array_equal(hm[b], orc.hmult_relin_level(ct1[b], ct2[b], key, P)), (ell, b)
            assert np.array_equal(hr[b], orc.hrot_level(ct1[b], g, key, P)), (ell, b)
        pt = synth.uniform_residues(rng, list(q) + list(ps.p_primes), ps.N, lead=(2,))
        dh = host(ctx.hrot_dh_mac(dev(ct1[0]), [g, 1], [d_key, d_key], dev(pt), level=ell))
        assert np.array_equal(dh, orc.hrot_dh_mac_level(ct1[0], [g, 1], [key, key], pt, P)), ell
        assert np.array_equal(host(ctx.rescale(ell, dev(ct1))), orc.rescale(ct1, P)), ell


def _random_case(seed, max_L=10, max_K=8):
    rng = np.random.default_rng(seed)
    logN = int(rng.choice([12, 12, 13]))
    L = int(rng.integers(1, max_L + 1))
    dnum = int(rng.choice([d for d in range(1, L + 1) if -(-L // -(-L // d)) == d and -(-L // d) <= 16]))
    K = int(rng.integers(1, max_K + 1))
    bits = [30, 36, 44, 49, 55, 59]
    qf = [int(rng.choice(bits)) for _ in range(L)]
    pf = [int(rng.choice([36, 49, 59, 60])) for _ in range(K)]
    return logN, qf, pf, dnum


@pytest.mark.parametrize("seed", list(range(40)) + [100 + i for i in range(8)])
def test_random_chains_levels_and_operations(orc, seed):
    """Seeded random parameter sets (1..10 limbs of 30..60 bits in any order, 1..8 special limbs, any digit
    count; seeds from 100 on: up to 32 limbs and 16 special limbs, digits of up to 16 limbs), a random level,
    every composed operation once; odd seeds with the library's second stream on."""
    logN, qf, pf, dnum = _random_case(500 + seed) if seed < 100 else _random_case(500 + seed, 32, 16)
    ps = synth.mixed_params(logN, qf, pf, dnum, "random%d" % seed)
    _say("seed", seed, "logN", logN, "q bits", qf, "p bits", pf, "dnum", dnum)
    _every_composed_operation_once(orc, ps, seed)


def _edge_case(seed):
    """Primes drawn from the edges of what a context accepts: the smallest = 1 mod 2N, either side of 2^28 (below it
    a conversion target is converted with integers), either side of 3*2^48 (the FP64 / integer bound), 53-54 bits,
    and just below 2^61."""
    rng = np.random.default_rng(47000 + seed)
    logN = int(rng.choice([12, 12, 13, 14]))
    floors = [logN + 1, logN + 2, 17, 20, 24, (1 << 28) - (1 << 20), (1 << 28) + 1, 31, 32, 33, 40,
              FP_LIMIT - (1 << 24), FP_LIMIT - (1 << 40), FP_LIMIT, FP_LIMIT + (1 << 30), 50, 52, 53, 54, 60,
              (1 << 61) - (1 << 26), (1 << 61) - (1 << 40)]
    L, K = int(rng.integers(1, 9)), int(rng.integers(1, 6))
    dnum = int(rng.choice([d for d in range(1, L + 1) if -(-L // -(-L // d)) == d]))
    qf = [int(floors[i]) for i in rng.integers(0, len(floors), size=L)]
    pf = [int(floors[i]) for i in rng.integers(0, len(floors), size=K)]
    return logN, qf, pf, dnum


@pytest.mark.parametrize("seed", range(16))
def test_primes_at_the_edges_of_the_accepted_range(orc, seed):
    logN, qf, pf, dnum = _edge_case(seed)
    ps = synth.mixed_params(logN, qf, pf, dnum, "edge%d" % seed)
    assert all(p < 1 << 61 for p in ps.primes)
    _say("seed", seed, "logN", logN, "prime bits", [p.bit_length() for p in ps.primes], "dnum", dnum)
    _every_composed_operation_once(orc, ps, seed, corners=True)


def _every_composed_operation_once(orc, ps, seed, corners=False):
    logN = ps.logN
    from paper_2310_16530_amd import binding
    ctx = binding.Context(ps.logN, ps.L, ps.K, ps.dnum, ps.primes)     # not cached: every seed has its own chain
    ctx.set_overlap(seed % 2 == 1)
    P = orc.Params(ps.logN, ps.L, ps.K, ps.dnum, ps.primes)
    rng = np.random.default_rng(900 + seed)
    N = ps.N
    ell = int(rng.integers(1, ps.L + 1))
    q = ps.q_primes[:ell]
    key = synth.uniform_residues(rng, ps.primes, N, lead=(ps.dnum, 2))
    d_key = dev(key)
    ct1 = synth.uniform_residues(rng, q, N, lead=(2, 2))
    ct2 = synth.uniform_residues(rng, q, N, lead=(2, 2))
    if corners:  # extreme residues against each other in every limb, also in the key
        for i, p in enumerate(q):
            ct1[0, :, i, :6] = [0, 1, p - 1, p - 2, p // 2, p // 2 + 1]
            ct2[0, :, i, :6] = [p - 1, p - 1, p - 1, 0, p // 2, 1]
        for i, p in enumerate(ps.primes):
            key[:, :, i, :3] = [p - 1, 0, 1]
        d_key = dev(key)
    g = synth.galois_element(int(rng.integers(1, 100)), logN)
    hm = host(ctx.hmult_relin_at(ell, dev(ct1), dev(ct2), d_key))
    hr = host(ctx.hrot_at(ell, dev(ct1), g, d_key))
    for b in range(2):
        assert np.array_equal(hm[b], orc.hmult_relin_level(ct1[b], ct2[b], key, P)), ("hmult", ell, b)
        assert np.array_equal(hr[b], orc.hrot_level(ct1[b], g, key, P)), ("hrot", ell, b)
    gs = [g, 1, synth.galois_element(-1, logN)]
    basis = list(q) + list(ps.p_primes)
    pt = synth.uniform_residues(rng, basis, N, lead=(len(gs),))
    d_keys = [d_key] * len(gs)
    keys = [key] * len(gs)
    assert np.array_equal(host(ctx.hrot_hoisted_mac_at(ell, dev(ct1[0]), gs, d_keys, dev(pt[:, :ell]))),
                          orc.hrot_hoisted_mac_level(ct1[0], gs, keys, np.ascontiguousarray(pt[:, :ell]), P)), ("hoisted", ell)
    assert np.array_equal(host(ctx.hrot_dh_mac(dev(ct1[0]), gs, d_keys, dev(pt), level=ell)),
                          orc.hrot_dh_mac_level(ct1[0], gs, keys, pt, P)), ("double hoisted", ell)
    if ell >= 2:
        assert np.array_equal(host(ctx.rescale(ell, dev(ct1))), orc.rescale(ct1, P)), ("rescale", ell)
        mr = host(ctx.hmult_relin_rescale_at(ell, dev(ct1), dev(ct2), d_key))
        for b in range(2):
            assert np.array_equal(mr[b], orc.hmult_relin_rescale_level(ct1[b], ct2[b], key, P)), ("merged", ell, b)
        assert np.array_equal(host(ctx.hrot_dh_mac_rescale_at(ell, dev(ct1[0]), gs, d_keys, dev(pt))),
                              orc.hrot_dh_mac_rescale_level(ct1[0], gs, keys, pt, P)), ("merged dh", ell)


def test_sixteen_rotations_in_one_launch_near_the_fp64_prime_limit(orc):
    """A full chunk of rotations accumulated in the final kernel with primes just below 3*2^48: the FP64
    accumulators must be folded often enough to stay exact."""
    ps = synth.mixed_params(12, [FP_LIMIT - (1 << 24)] * 4, [59, 59], 2, "fp_limit")
    assert all(p < FP_LIMIT for p in ps.q_primes)
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = np.random.default_rng(77)
    n_rot = 16
    gs = [synth.galois_element(r, ps.logN) for r in range(1, n_rot + 1)]
    rks = [synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2)) for _ in gs]
    ct = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(2,))
    pt = synth.uniform_residues(rng, ps.primes, ps.N, lead=(n_rot,))
    for p_i, p in enumerate(ps.primes):          # worst case for the accumulators: operands at the top of the range
        pt[:, p_i, :64] = p - 1
    d_rks = [dev(k) for k in rks]
    got = host(ctx.hrot_hoisted_mac(dev(ct), gs, d_rks, dev(np.ascontiguousarray(pt[:, :ps.L]))))
    assert np.array_equal(got, orc.hrot_hoisted_mac(ct, gs, rks, np.ascontiguousarray(pt[:, :ps.L]), P))
    got = host(ctx.hrot_dh_mac(dev(ct), gs, d_rks, dev(pt)))
    assert np.array_equal(got, orc.hrot_dh_mac_level(ct, gs, rks, pt, P))


def test_wide_digits_at_the_top_of_the_fp64_range(orc):
    """Digits and a special basis of 16 limbs with q-limbs just below 3*2^48, and coefficients chosen so that
    every pre-multiplied source of the ModUp conversion is q_i - 1: the FP64 accumulators of the fused conversions
    see the largest terms their bounds allow, over two rounds of 8 sources."""
    ps = synth.mixed_params(12, [FP_LIMIT - (1 << 24)] * 16, [60] * 16, 1, "wide_fp_limit")
    assert all(p < FP_LIMIT for p in ps.q_primes) and ps.L // ps.dnum == 16
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = np.random.default_rng(78)
    N, L = ps.N, ps.L
    x = synth.uniform_residues(rng, ps.q_primes, N, lead=())
    Q = 1
    for q in ps.q_primes:
        Q *= q
    for i, q in enumerate(ps.q_primes):
        qhat = (Q // q) % q
        x[i, :64] = (q - 1) * qhat % q          # y_i = x_i * qhat^-1 = q_i - 1
        x[i, 64:128] = qhat                      # y_i = 1
    d = np.stack([orc.ntt(x[i], ps.logN, ps.q_primes[i], P.psi[i]) for i in range(L)])
    key = synth.uniform_residues(rng, ps.primes, N, lead=(ps.dnum, 2))
    for p_i, p in enumerate(ps.primes):
        key[:, :, p_i, :32] = p - 1
    got = host(ctx.keyswitch_at(L, dev(d[None]), dev(key)))[0]
    assert np.array_equal(got, orc.keyswitch_level(d, key, P))
    ct = np.stack([d, d])
    assert np.array_equal(host(ctx.hmult_relin_rescale_at(L, dev(ct[None]), dev(ct[None]), dev(key)))[0],
                          orc.hmult_relin_rescale_level(ct, ct, key, P))


@pytest.mark.parametrize("name,shape", [("fp64_special", (12, [44, 36, 55, 30, 55, 59, 30, 55], [49, 49, 49, 36], 4)),
                                        ("mixed_special", (13, [50, 58, 44, 59], [59, 49, 36], 2))])
def test_second_stream_with_fp64_special_limbs(orc, name, shape):
    """With the library's second stream on, the FP64 ModUp conversion runs beside the inner product on the limbs that
    feed the ModDown.  When some of those limbs are FP64 primes themselves (special primes below 3*2^48) the inner
    product needs that conversion's output and has to wait for it: every key-switch entry point, several times in a
    row, against the oracle."""
    logN, qf, pf, dnum = shape
    ps = synth.mixed_params(logN, qf, pf, dnum, name)
    assert any(p < FP_LIMIT for p in ps.p_primes) and any(p >= FP_LIMIT for p in ps.q_primes)
    from paper_2310_16530_amd import binding
    ctx = binding.Context(ps.logN, ps.L, ps.K, ps.dnum, ps.primes)
    ctx.set_overlap(True)
    P = orc.Params(ps.logN, ps.L, ps.K, ps.dnum, ps.primes)
    rng = np.random.default_rng(77 + logN)
    N = ps.N
    key = synth.uniform_residues(rng, ps.primes, N, lead=(ps.dnum, 2))
    d_key = dev(key)
    g = synth.galois_element(3, logN)
    for ell in (ps.L, ps.L - 1):
        q = ps.q_primes[:ell]
        ct1 = synth.uniform_residues(rng, q, N, lead=(4, 2))
        ct2 = synth.uniform_residues(rng, q, N, lead=(4, 2))
        want = [np.stack([orc.keyswitch_level(ct1[b, 0], key, P) for b in range(4)]),
                np.stack([orc.hmult_relin_level(ct1[b], ct2[b], key, P) for b in range(4)]),
                np.stack([orc.hrot_level(ct1[b], g, key, P) for b in range(4)]),
                np.stack([orc.hmult_relin_rescale_level(ct1[b], ct2[b], key, P) for b in range(4)])]
        d1, d2, d0 = dev(ct1), dev(ct2), dev(ct1[:, 0])
        for rep in range(3):
            _say(name, "level", ell, "repetition", rep)
            got = [host(ctx.keyswitch_at(ell, d0, d_key)), host(ctx.hmult_relin_at(ell, d1, d2, d_key)),
                   host(ctx.hrot_at(ell, d1, g, d_key)), host(ctx.hmult_relin_rescale_at(ell, d1, d2, d_key))]
            for what, a, b in zip(("keyswitch", "hmult", "hrot", "merged"), got, want):
                assert np.array_equal(a, b), (what, ell, rep)
