"""Parity of the HIP path against the CPU oracle, bit for bit, through the C ABI (needs an MI355X).

Every comparison is exact (integer work): `np.array_equal` on the uint64 words.
Sizes: reduced shapes of the same family that the oracle finishes in seconds (several
workgroup tiles, every supported ring degree, digit sizes 1..16), then the full workload
shapes in the launch configuration the benchmark times.
"""
import numpy as np
import pytest

from paper_2310_16530_amd import synth

pytestmark = pytest.mark.gpu


def _torch():
    import torch
    return torch


def dev(a):
    torch = _torch()
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int64)).to("cuda:0")


def host(t):
    return t.cpu().numpy().view(np.uint64)


def say(*a):
    """progress line, flushed: names the case before each long step"""
    print(*a, flush=True)


_CTX = {}


def gpu_ctx(ps):
    from paper_2310_16530_amd import binding
    key = (ps.logN, ps.L, ps.K, ps.dnum, ps.primes)
    if key not in _CTX:
        _CTX[key] = binding.Context(ps.logN, ps.L, ps.K, ps.dnum, ps.primes)
    return _CTX[key]


_ORC = {}


def orc_params(orc, ps):
    key = (ps.logN, ps.L, ps.K, ps.dnum, ps.primes)
    if key not in _ORC:
        _ORC[key] = orc.Params.from_set(ps)
    return _ORC[key]


def test_library_is_the_hip_one_and_roots_agree(orc):
    from paper_2310_16530_amd import binding
    lib = binding.load()
    assert lib._name.endswith("libckks_mi355x.so")
    ps = synth.CFG0
    ctx = gpu_ctx(ps)
    P = orc_params(orc, ps)
    assert [ctx.psi(i) for i in range(ps.L + ps.K)] == P.psi


# ------------------------------------------------------------------------------ NTT
@pytest.mark.parametrize("logN", [12, 13, 14, 15, 16])
def test_ntt_intt_parity_all_ring_degrees(orc, logN):
    # 3 fifty-bit limbs + 2 sixty-bit limbs, batch 3: 15 limb jobs, up to 16 tiles each
    ps = synth.small_params(logN, 3, 2, 3)
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = np.random.default_rng(100 + logN)
    x = synth.uniform_residues(rng, ps.primes, ps.N, lead=(3,))
    x[0, :, :7] = 0
    for i, p in enumerate(ps.primes):       # edge values: zeros and q-1 runs
        x[1, i, :] = p - 1
    x[2, 0, :] = 0
    fwd = host(ctx.ntt(dev(x)))
    assert np.array_equal(fwd, orc.ntt_batch(x, P, 0))
    inv = host(ctx.intt(dev(x)))
    assert np.array_equal(inv, orc.ntt_batch(x, P, 0, inverse=True))
    back = host(ctx.intt(ctx.ntt(dev(x))))
    assert np.array_equal(back, x)
    # sub-range of the chain: limbs 2..4 only (prime_first = 2), single batch, single limb
    sub = np.ascontiguousarray(x[0, 2:5])
    assert np.array_equal(host(ctx.ntt(dev(sub), prime_first=2)),
                          np.stack([orc.ntt(sub[i], logN, ps.primes[2 + i], P.psi[2 + i]) for i in range(3)]))
    one = np.ascontiguousarray(x[0, 4:5])
    assert np.array_equal(host(ctx.intt(dev(one), prime_first=4))[0], orc.intt(one[0], logN, ps.primes[4], P.psi[4]))


@pytest.mark.timeout(900)
def test_ntt_config1_full_size(orc):
    """workload 1: 16 polynomials x 24 fifty-bit limbs at N = 2^16, forward, inverse, round trip."""
    ps = synth.CFG1
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    x = synth.uniform_residues(synth.rng_for(1, 0), ps.primes, ps.N, lead=(synth.CFG1_BATCH,))
    d = dev(x)
    ctx.ntt(d)
    assert np.array_equal(host(d), orc.ntt_batch(x, P, 0))
    # definition, sampled slots (independent of the oracle's fast network)
    got = host(d)
    for (b, l, j) in [(0, 0, 0), (3, 7, 12345), (15, 23, 65535)]:
        assert int(got[b, l, j]) == orc.ntt_def_at(x[b, l], 16, ps.primes[l], P.psi[l], j)
    ctx.intt(d)
    assert np.array_equal(host(d), x)
    d2 = dev(x)
    ctx.intt(d2)
    assert np.array_equal(host(d2), orc.ntt_batch(x, P, 0, inverse=True))


# ------------------------------------------------------------------ base conversion
CONV_SHAPES = [(12, 4, 2, 2), (12, 3, 1, 3), (13, 6, 3, 2), (12, 8, 8, 1), (14, 6, 6, 1), (12, 10, 5, 2),
               (12, 7, 7, 1), (12, 8, 4, 2), (12, 9, 9, 1), (12, 12, 12, 1), (12, 16, 16, 1), (12, 20, 10, 2),
               (12, 5, 3, 2), (12, 7, 3, 3), (12, 10, 4, 4), (12, 19, 10, 2)]   # last four: dnum does not divide L


@pytest.mark.parametrize("shape", CONV_SHAPES)
def test_modup_moddown_parity(orc, shape):
    ps = synth.small_params(*shape)
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = np.random.default_rng(sum(shape))
    x = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(2,))
    x[0, :, 0] = 0
    for i, p in enumerate(ps.q_primes):
        x[0, i, 1] = p - 1
    up = host(ctx.modup(dev(x)))
    for b in range(2):
        assert np.array_equal(up[b], orc.modup(x[b], P))
    y = synth.uniform_residues(rng, ps.primes, ps.N, lead=(2,))
    for i, p in enumerate(ps.primes):
        y[1, i, 5] = p - 1
    down = host(ctx.moddown(dev(y)))
    for b in range(2):
        assert np.array_equal(down[b], orc.moddown(y[b], P))


@pytest.mark.timeout(900)
def test_modup_moddown_full_size(orc):
    ps = synth.CFG2
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = synth.rng_for(2, 7)
    x = synth.uniform_residues(rng, ps.q_primes, ps.N)
    assert np.array_equal(host(ctx.modup(dev(x))), orc.modup(x, P))
    y = synth.uniform_residues(rng, ps.primes, ps.N)
    assert np.array_equal(host(ctx.moddown(dev(y))), orc.moddown(y, P))


# --------------------------------------------------------------------- automorphism
@pytest.mark.parametrize("logN", [12, 16])
def test_automorph_parity(orc, logN):
    ps = synth.small_params(logN, 2, 1, 2)
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = np.random.default_rng(logN)
    x = synth.uniform_residues(rng, ps.primes, ps.N, lead=(2,))
    x[0, 0, :3] = 0
    for g in [1, 5, 25, synth.galois_element(-1, logN), synth.galois_element(7, logN), 2 * ps.N - 1, 3]:
        for ev in (False, True):
            got = host(ctx.automorph(dev(x), g, ev))
            assert np.array_equal(got, orc.automorph_limbs(x, P, 0, g, ev)), (g, ev)


# ------------------------------------------------- key switch, HMult, HRot (reduced shapes)
def make_keys(orc, ps, P, rng, s_hat, sp_hat):
    a = synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum,))
    e = synth.gaussian_error(rng, (ps.dnum, ps.N))
    return orc.make_switch_key(s_hat, sp_hat, a, e, P)


def _orc_pointwise(orc, op, a, b, primes):
    """a [batch][n][N], b [period][n][N] -> [batch][n][N]; MAC is expressed by the caller (mul then add)."""
    return np.stack([orc.pointwise(op, a[g], b[g % b.shape[0]], primes) for g in range(a.shape[0])])


@pytest.mark.parametrize("shape,prime_first,n_limbs", [((12, 4, 2, 2), 0, 6), ((13, 6, 3, 2), 2, 5), ((16, 3, 1, 3), 1, 3)])
def test_pointwise_parity(orc, shape, prime_first, n_limbs):
    from paper_2310_16530_amd import binding
    ps = synth.small_params(*shape)
    ctx = gpu_ctx(ps)
    primes = ps.primes[prime_first:prime_first + n_limbs]
    rng = np.random.default_rng(77 + sum(shape) + prime_first)
    a = synth.uniform_residues(rng, primes, ps.N, lead=(6,))
    b = synth.uniform_residues(rng, primes, ps.N, lead=(6,))
    c = synth.uniform_residues(rng, primes, ps.N, lead=(6,))
    for i, q in enumerate(primes):  # corners: 0, 1, q-1 against each other
        a[0, i, :9] = [0, 0, 0, 1, 1, q - 1, q - 1, q - 1, q - 2]
        b[0, i, :9] = [0, 1, q - 1, 1, q - 1, q - 1, 1, 0, q - 2]
    da, db, dc = dev(a), dev(b), dev(c)
    for period in (6, 1, 2, 4):  # 4 does not divide the batch: the second operand wraps around
        bb = b[:period]
        dbb = db[:period].contiguous()
        for op, name in ((binding.PW_ADD, "add"), (binding.PW_SUB, "sub"), (binding.PW_MUL, "mul")):
            want = _orc_pointwise(orc, name, a, bb, primes)
            assert np.array_equal(host(ctx.pointwise(op, da, dbb, prime_first=prime_first)), want), (name, period)
        acc = dc.clone()
        ctx.pointwise(binding.PW_MAC, da, dbb, out=acc, prime_first=prime_first)
        want = _orc_pointwise(orc, "add", _orc_pointwise(orc, "mul", a, bb, primes), c, primes)
        assert np.array_equal(host(acc), want), ("mac", period)
    # in place on the first operand, and on the second when the operands pair one to one
    x = da.clone()
    ctx.pointwise(binding.PW_MUL, x, db, out=x, prime_first=prime_first)
    assert np.array_equal(host(x), _orc_pointwise(orc, "mul", a, b, primes))
    y = db.clone()
    ctx.pointwise(binding.PW_SUB, da, y, out=y, prime_first=prime_first)
    assert np.array_equal(host(y), _orc_pointwise(orc, "sub", a, b, primes))


KS_SHAPES = [(12, 4, 2, 2), (12, 3, 1, 3), (13, 6, 3, 2), (12, 6, 6, 1), (14, 4, 2, 2), (12, 14, 7, 2), (12, 8, 8, 1),
             (12, 20, 1, 20), (15, 2, 2, 1), (12, 9, 9, 1), (12, 12, 12, 1), (12, 32, 16, 2),
             (12, 5, 3, 2), (13, 7, 3, 3), (12, 10, 4, 4), (12, 23, 6, 4)]   # last four: dnum does not divide L


@pytest.mark.parametrize("shape", KS_SHAPES)
def test_keyswitch_hmult_hrot_parity_reduced(orc, shape):
    ps = synth.small_params(*shape)
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = np.random.default_rng(1000 + sum(shape))
    s = synth.ternary_hamming(rng, ps.N, 64)
    s_hat = orc.secret_eval(s, P)
    s2_hat = orc.pointwise("mul", s_hat, s_hat, ps.primes)
    evk = make_keys(orc, ps, P, rng, s_hat, s2_hat)
    d_evk = dev(evk)
    B = 3
    d = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(B,))
    d[2] = 0
    ks = host(ctx.keyswitch(dev(d), d_evk))
    for b in range(B):
        assert np.array_equal(ks[b], orc.keyswitch(d[b], evk, P)), b
    # decrypt-and-bound on the GPU result itself
    bound = orc.keyswitch_noise_bound(P, int(np.abs(s).sum()))
    assert np.abs(orc.keyswitch_noise(d[0], ks[0], s_hat, s2_hat, P)).max() <= bound

    ct1 = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(B, 2))
    ct2 = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(B, 2))
    hm = host(ctx.hmult_relin(dev(ct1), dev(ct2), d_evk))
    for b in range(B):
        assert np.array_equal(hm[b], orc.hmult_relin(ct1[b], ct2[b], evk, P)), b

    for rot in (1, -1):
        g = synth.galois_element(rot, ps.logN)
        sg_hat = orc.automorph_limbs(s_hat, P, 0, g, True)
        rk = make_keys(orc, ps, P, rng, s_hat, sg_hat)
        hr = host(ctx.hrot(dev(ct1), g, dev(rk)))
        for b in range(B):
            assert np.array_equal(hr[b], orc.hrot(ct1[b], g, rk, P)), (rot, b)


@pytest.mark.parametrize("shape", [(13, 4, 2, 2), (16, 3, 1, 3)])
def test_hrot_other_galois_elements(orc, shape):
    """Rotations gather their source rows whole and permute them on chip; the row-to-row property that rests on holds for
    every odd Galois element, so the conjugation, 3 (neither a power of 5 times a sign we use elsewhere) and far
    rotations are compared with the oracle too, singly and inside a hoisted rotate-MAC."""
    ps = synth.small_params(*shape)
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = np.random.default_rng(4242 + sum(shape))
    ct = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(2, 2))
    gs = [2 * ps.N - 1, 3, 2 * ps.N - 3, synth.galois_element(ps.N // 2 - 1, ps.logN), synth.galois_element(1000, ps.logN)]
    rks = [synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2)) for _ in gs]
    d_ct = dev(ct)
    for g, rk in zip(gs, rks):
        say("hrot with Galois element", g)
        got = host(ctx.hrot(d_ct, g, dev(rk)))
        for b in range(2):
            assert np.array_equal(got[b], orc.hrot(ct[b], g, rk, P)), (g, b)
    pt = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(len(gs),))
    got = host(ctx.hrot_hoisted_mac(dev(ct[0]), gs, [dev(r) for r in rks], dev(pt)))
    assert np.array_equal(got, orc.hrot_hoisted_mac(ct[0], gs, rks, pt, P))


@pytest.mark.parametrize("shape,n_rot", [((12, 4, 2, 2), 3), ((13, 6, 3, 2), 11), ((12, 3, 1, 3), 8), ((12, 6, 6, 1), 9),
                                         ((12, 7, 3, 3), 5)])
def test_hoisted_mac_parity_reduced(orc, shape, n_rot):
    ps = synth.small_params(*shape)
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = np.random.default_rng(2000 + sum(shape))
    s = synth.ternary_hamming(rng, ps.N, 64)
    s_hat = orc.secret_eval(s, P)
    rots = [1, 2, 3, 4, 5, 6, 7, 8, 16, -1, 32][:n_rot]
    gs = [synth.galois_element(r, ps.logN) for r in rots]
    rks = [make_keys(orc, ps, P, rng, s_hat, orc.automorph_limbs(s_hat, P, 0, g, True)) for g in gs]
    ct = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(2,))
    pt = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(n_rot,))
    d_rks = [dev(k) for k in rks]
    got = host(ctx.hrot_hoisted_mac(dev(ct), gs, d_rks, dev(pt)))
    # unit plaintext on one rotation reproduces that rotated ciphertext; decrypt-and-bound it
    r = n_rot - 1
    unit = np.zeros_like(pt)
    unit[r] = 1
    Rr = host(ctx.hrot_hoisted_mac(dev(ct), gs, d_rks, dev(unit)))
    if ps.L % ps.dnum == 0:
        want, per = orc.hrot_hoisted_mac(ct, gs, rks, pt, P, want_per_rotation=True)
        assert np.array_equal(Rr, per[r])
    else:  # the oracle gives per-rotation outputs for digits of equal size only
        want = orc.hrot_hoisted_mac(ct, gs, rks, pt, P)
        assert np.array_equal(Rr, orc.hrot_hoisted_mac(ct, gs, rks, unit, P))
    assert np.array_equal(got, want)
    q = ps.q_primes
    sq = s_hat[:ps.L]

    def dec(c):
        return orc.pointwise("add", c[0], orc.pointwise("mul", c[1], sq, q), q)

    E = orc.centred_small(orc.pointwise("sub", dec(Rr), orc.automorph_limbs(dec(ct), P, 0, gs[r], True), q), P, ps.L)
    assert np.abs(E).max() <= orc.keyswitch_noise_bound(P, int(np.abs(s).sum()))


# ------------------------------------------------------------- full workload shapes
def test_config0_hmult_exact_shape(orc):
    ps = synth.CFG0
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = synth.rng_for(0, 0)
    s = synth.ternary_iid(rng, ps.N)
    s_hat = orc.secret_eval(s, P)
    s2_hat = orc.pointwise("mul", s_hat, s_hat, ps.primes)
    evk = make_keys(orc, ps, P, rng, s_hat, s2_hat)
    ct1 = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(2,))
    ct2 = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(2,))
    got = host(ctx.hmult_relin(dev(ct1), dev(ct2), dev(evk)))
    assert np.array_equal(got, orc.hmult_relin(ct1, ct2, evk, P))
    q = ps.q_primes
    sq = s_hat[:ps.L]

    def dec(c):
        return orc.pointwise("add", c[0], orc.pointwise("mul", c[1], sq, q), q)

    E = orc.centred_small(orc.pointwise("sub", dec(got), orc.pointwise("mul", dec(ct1), dec(ct2), q), q), P, ps.L)
    assert np.abs(E).max() <= orc.keyswitch_noise_bound(P, int(np.abs(s).sum()))


@pytest.mark.timeout(900)
def test_config2_hmult_batch8_full_size(orc):
    """workload 2 in the benchmark's launch configuration (batch 8, shared evk): all eight products are
    compared with the oracle word for word and checked by decrypt-and-bound."""
    ps = synth.CFG2
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = synth.rng_for(2, 0)
    s = synth.ternary_hamming(rng, ps.N, 192)
    s_hat = orc.secret_eval(s, P)
    s2_hat = orc.pointwise("mul", s_hat, s_hat, ps.primes)
    evk = make_keys(orc, ps, P, rng, s_hat, s2_hat)
    B = synth.CFG2_BATCH
    ct1 = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(B, 2))
    ct2 = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(B, 2))
    d1, d2, dk = dev(ct1), dev(ct2), dev(evk)
    got = host(ctx.hmult_relin(d1, d2, dk))
    for b in range(B):
        say("cfg2 hmult: oracle pair", b)
        assert np.array_equal(got[b], orc.hmult_relin(ct1[b], ct2[b], evk, P)), b
    # the launch configuration bench.py times: the library's second stream on, calls back to back
    ctx.set_overlap(True)
    try:
        for _ in range(3):
            assert np.array_equal(host(ctx.hmult_relin(d1, d2, dk)), got)
    finally:
        ctx.set_overlap(False)
    q = ps.q_primes
    sq = s_hat[:ps.L]
    bound = orc.keyswitch_noise_bound(P, 192)
    assert bound <= 1160  # ceil(2^-29) + 6*193 + 1

    def dec(c):
        return orc.pointwise("add", c[0], orc.pointwise("mul", c[1], sq, q), q)

    for b in range(B):
        E = orc.centred_small(orc.pointwise("sub", dec(got[b]), orc.pointwise("mul", dec(ct1[b]), dec(ct2[b]), q), q), P, ps.L)
        assert np.abs(E).max() <= bound, b


@pytest.mark.timeout(900)
def test_config2_hrot_and_keyswitch_full_size(orc):
    ps = synth.CFG2
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = synth.rng_for(2, 1)
    B = synth.CFG2_BATCH
    # parity needs no structured key: uniform residues stand in for the key limbs
    rk = synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2))
    ct = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(B, 2))
    g = synth.galois_element(1, ps.logN)
    dct, drk = dev(ct), dev(rk)
    got = host(ctx.hrot(dct, g, drk))
    for b in range(B):
        say("cfg2 hrot: oracle ciphertext", b)
        assert np.array_equal(got[b], orc.hrot(ct[b], g, rk, P)), b
    ctx.set_overlap(True)  # as bench.py runs it
    try:
        for _ in range(3):
            assert np.array_equal(host(ctx.hrot(dct, g, drk)), got)
    finally:
        ctx.set_overlap(False)
    d = np.ascontiguousarray(ct[:2, 1])
    ks = host(ctx.keyswitch(dev(d), dev(rk)))
    for b in range(2):
        assert np.array_equal(ks[b], orc.keyswitch(d[b], rk, P)), b


@pytest.mark.timeout(900)
def test_config3_rotate_and_sum_full_size(orc):
    """workload 3: one ciphertext, the 17 listed offsets, hoisted ModUp, plaintext MAC."""
    ps = synth.CFG3
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = synth.rng_for(3, 0)
    gs = [synth.galois_element(r, ps.logN) for r in synth.CFG3_ROTATIONS]
    n_rot = len(gs)
    assert n_rot == 17
    rks = [synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2)) for _ in gs]
    ct = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(2,))
    pt = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(n_rot,))
    got = host(ctx.hrot_hoisted_mac(dev(ct), gs, [dev(k) for k in rks], dev(pt)))
    assert np.array_equal(got, orc.hrot_hoisted_mac(ct, gs, rks, pt, P))


@pytest.mark.timeout(900)
def test_config4_coeff_to_slot_shape_full_size(orc):
    """workload 4: L=35, K=7, dnum=5, 32 rotations +-2^i (the identity element g = 1 from +-2^15 included):
    the 32-rotation call (two launches' worth of rotations) is compared with the oracle word for word.
    Extra, not the parity evidence: a sub-list gives the oracle's result too, and the call is linear in
    the rotation list."""
    ps = synth.CFG4
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = synth.rng_for(4, 0)
    gs = [synth.galois_element(r, ps.logN) for r in synth.CFG4_ROTATIONS]
    assert len(gs) == 32 and gs[30] == 1 and gs[31] == 1
    ct = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(2,))
    d_ct = dev(ct)
    rks = [dev(synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2))) for _ in gs]
    pt = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(32,))
    d_pt = dev(pt)
    full = host(ctx.hrot_hoisted_mac(d_ct, gs, rks, d_pt))
    say("cfg4: oracle, 32 rotations")
    assert np.array_equal(full, orc.hrot_hoisted_mac(ct, gs, [host(k) for k in rks], pt, P))
    sub = [0, 1, 29, 30, 31]
    want = orc.hrot_hoisted_mac(ct, [gs[i] for i in sub], [host(rks[i]) for i in sub], np.ascontiguousarray(pt[sub]), P)
    got_sub = host(ctx.hrot_hoisted_mac(d_ct, [gs[i] for i in sub], [rks[i] for i in sub], dev(np.ascontiguousarray(pt[sub]))))
    assert np.array_equal(got_sub, want)
    acc = np.zeros_like(full)
    for c in range(4):
        part = host(ctx.hrot_hoisted_mac(d_ct, gs[8 * c:8 * c + 8], rks[8 * c:8 * c + 8], d_pt[8 * c:8 * c + 8].contiguous()))
        for t in range(2):
            acc[t] = orc.pointwise("add", acc[t], part[t], ps.q_primes)
    assert np.array_equal(full, acc)


@pytest.mark.timeout(900)
def test_config4_double_hoisted_full_size(orc):
    """workload 4's shape through the double-hoisted call: all 32 rotations against the oracle, word for word."""
    ps = synth.CFG4
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = synth.rng_for(4, 3)
    gs = [synth.galois_element(r, ps.logN) for r in synth.CFG4_ROTATIONS]
    ct = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(2,))
    rks = [synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2)) for _ in gs]
    pt = synth.uniform_residues(rng, ps.primes, ps.N, lead=(32,))
    say("cfg4 double hoisting: gpu")
    got = host(ctx.hrot_dh_mac(dev(ct), gs, [dev(k) for k in rks], dev(pt)))
    say("cfg4 double hoisting: oracle")
    assert np.array_equal(got, orc.hrot_dh_mac_level(ct, gs, rks, pt, P))


# ------------------------------------------------------------ error paths on a live context
def test_error_paths_return_codes_without_launching(orc):
    import ctypes
    from paper_2310_16530_amd import binding
    torch = _torch()
    lib = binding.load()
    ps = synth.small_params(12, 4, 2, 2)
    ctx = gpu_ctx(ps)
    x = torch.zeros((2, ps.L, ps.N), dtype=torch.int64, device="cuda:0")
    key = torch.zeros((ps.dnum, 2, ps.L + ps.K, ps.N), dtype=torch.int64, device="cuda:0")
    ws = ctx.workspace(binding.OP_HROT, 1)
    h, p = ctx.handle, x.data_ptr()
    assert lib.ckks_ntt(h, None, 0, 1, 1, None) == binding.CKKS_EINVAL
    assert lib.ckks_ntt(h, p + 8, 0, 1, 1, None) == binding.CKKS_EINVAL             # misaligned
    assert lib.ckks_ntt(h, p, 5, 2, 1, None) == binding.CKKS_EINVAL                 # beyond the prime chain
    assert lib.ckks_ntt(h, p, 0, 0, 1, None) == binding.CKKS_EINVAL
    assert b"prime chain" in lib.ckks_last_error(h) or b"positive" in lib.ckks_last_error(h)
    assert lib.ckks_automorph(h, p, p, 0, 1, 5, 1, 1, None) == binding.CKKS_EINVAL  # in place
    out = torch.empty_like(x)
    assert lib.ckks_automorph(h, p, out.data_ptr(), 0, 1, 4, 1, 1, None) == binding.CKKS_EINVAL      # even g
    assert lib.ckks_automorph(h, p, out.data_ptr(), 0, 1, 2 * ps.N + 1, 1, 1, None) == binding.CKKS_EINVAL
    assert lib.ckks_hrot(h, p, 4, key.data_ptr(), out.data_ptr(), 1, ws.data_ptr(), ws.numel(), None) == binding.CKKS_EINVAL
    assert lib.ckks_hrot(h, p, 5, key.data_ptr(), out.data_ptr(), 1, ws.data_ptr(), 1024, None) == binding.CKKS_ENOMEM
    assert lib.ckks_hrot(h, p, 5, key.data_ptr(), out.data_ptr(), 1, None, 1 << 40, None) == binding.CKKS_EINVAL
    assert lib.ckks_hrot(h, p, 5, key.data_ptr(), out.data_ptr(), 0, ws.data_ptr(), ws.numel(), None) == binding.CKKS_EINVAL
    # outputs that share memory with an input, or a workspace that shares memory with an operand, are rejected
    ct = torch.zeros((2, 2, ps.L, ps.N), dtype=torch.int64, device="cuda:0")
    c0, c1, k, w, wn = ct[0].data_ptr(), ct[1].data_ptr(), key.data_ptr(), ws.data_ptr(), ws.numel()
    limb = ps.N * 8
    assert lib.ckks_hrot(h, c0, 5, k, c0, 1, w, wn, None) == binding.CKKS_EINVAL
    assert b"overlaps" in lib.ckks_last_error(h)
    assert lib.ckks_hrot(h, c0, 5, k, c0 + limb, 1, w, wn, None) == binding.CKKS_EINVAL           # partial overlap
    assert lib.ckks_hrot(h, c0, 5, k, c1, 1, w, wn, None) == binding.CKKS_OK                      # adjacent is fine
    assert lib.ckks_hmult_relin(h, c0, c1, k, c1, 1, w, wn, None) == binding.CKKS_EINVAL          # out is ct2
    assert lib.ckks_hmult_relin(h, c0, c1, k, c0, 1, w, wn, None) == binding.CKKS_EINVAL          # out is ct1
    assert lib.ckks_keyswitch(h, c0, k, c0, 1, w, wn, None) == binding.CKKS_EINVAL
    assert lib.ckks_hrot(h, w, 5, k, c1, 1, w, wn, None) == binding.CKKS_EINVAL                   # input inside the workspace
    assert lib.ckks_rescale(h, ps.L, c0, c0, 1, w, wn, None) == binding.CKKS_EINVAL
    gal = (ctypes.c_uint32 * 1)(5)
    kp = (ctypes.c_void_p * 1)(k)
    ptx = torch.zeros((1, ps.L + ps.K, ps.N), dtype=torch.int64, device="cuda:0")
    assert lib.ckks_hrot_hoisted_mac(h, c0, 1, gal, kp, ptx.data_ptr(), c0, w, wn, None) == binding.CKKS_EINVAL
    assert lib.ckks_hrot_hoisted_mac(h, c0, 1, gal, kp, c1, c1, w, wn, None) == binding.CKKS_EINVAL   # out is the plaintext
    assert lib.ckks_hrot_dh_mac(h, c0, 1, gal, kp, ptx.data_ptr(), c0, w, wn, None) == binding.CKKS_EINVAL
    assert lib.ckks_hrot_multi_at(h, ps.L, c0, gal, kp, c0, 1, w, wn, None) == binding.CKKS_EINVAL
    # the binding checks sizes the C ABI cannot see: a key without its special limbs, a short output
    short_key = torch.zeros((ps.dnum, 2, ps.L, ps.N), dtype=torch.int64, device="cuda:0")
    with pytest.raises(ValueError, match="rk: expected"):
        ctx.hrot(ct[0], 5, short_key)
    with pytest.raises(ValueError, match="out"):
        ctx.hrot(ct[0], 5, key, out=torch.zeros((2, ps.L - 1, ps.N), dtype=torch.int64, device="cuda:0"))
    with pytest.raises(ValueError, match="ct2"):
        ctx.hmult_relin(ct[0], ct[1][:1], key)
    with pytest.raises(ValueError, match="level"):
        ctx.hrot(ct[0], 5, key, level=ps.L + 1)
    o = out.data_ptr()
    assert lib.ckks_pointwise(h, 4, p, p, o, 0, 1, 1, 1, None) == binding.CKKS_EINVAL                # unknown op
    assert lib.ckks_pointwise(h, -1, p, p, o, 0, 1, 1, 1, None) == binding.CKKS_EINVAL
    assert lib.ckks_pointwise(h, binding.PW_ADD, p, p, o, 0, 1, 2, 3, None) == binding.CKKS_EINVAL   # period > batch
    assert lib.ckks_pointwise(h, binding.PW_ADD, p, p, o, 0, 1, 2, 0, None) == binding.CKKS_EINVAL
    assert lib.ckks_pointwise(h, binding.PW_ADD, p, None, o, 0, 1, 1, 1, None) == binding.CKKS_EINVAL
    assert lib.ckks_pointwise(h, binding.PW_ADD, p, p, o, 5, 2, 1, 1, None) == binding.CKKS_EINVAL   # beyond the chain
    n = ctypes.c_size_t()
    assert lib.ckks_workspace_bytes(h, 99, 1, ctypes.byref(n)) == binding.CKKS_EINVAL
    # transform-only context: key-switch entry points are unsupported, transforms work
    t_only = gpu_ctx(synth.small_params(12, 2, 0, 1))
    assert lib.ckks_modup(t_only.handle, p, out.data_ptr(), 1, None) == binding.CKKS_EUNSUPPORTED
    assert lib.ckks_workspace_bytes(t_only.handle, binding.OP_KEYSWITCH, 1, ctypes.byref(n)) == binding.CKKS_EUNSUPPORTED
    torch.cuda.synchronize()


def test_repeat_runs_are_bit_identical_and_profile_counts_launches(orc):
    ps = synth.small_params(13, 6, 3, 2)
    ctx = gpu_ctx(ps)
    rng = np.random.default_rng(9)
    ct = dev(synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(2, 2)))
    rk = dev(synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2)))
    g = synth.galois_element(3, ps.logN)
    first = host(ctx.hrot(ct, g, rk))
    ctx.profile_enable(True)
    for _ in range(3):
        assert np.array_equal(host(ctx.hrot(ct, g, rk)), first)
    prof = ctx.profile_read()
    ctx.profile_enable(False)
    # kernels are named as a profiler prints them; q-limbs run on the FP64 arithmetic, special limbs on integers
    # <.., rotation, not hoisted, fused>: the q-limb launch also ends the ModDown, so there is no kernel after it;
    # special limbs belong to no digit and run the plain variant <.., 0, false, false>
    assert prof["ks_inner_kernel<FpAr, 5, 2, false, true>"][0] == 3 and prof["ks_inner_kernel<IntAr, 5, 0, false, false>"][0] == 3
    assert not any(k.startswith("ks_final_kernel") for k in prof) and prof["inv_contig_kernel<FpAr, 5, 2>"][0] == 3
    # the ModDown conversion (2..8 sources) of FP64 targets runs on the matrix cores: <log2 N - 8, products, direction, ..>
    hits = [v for k, v in prof.items() if k.startswith("conv_mfma_kernel<5, ") and k.split(", ")[2] == "2"]
    assert len(hits) == 1 and hits[0][0] == 3
    assert prof["conv_fwd_strided_kernel<FpAr, 5, 1, 3, false>"][0] == 3 and prof["conv_fwd_strided_kernel<IntAr, 5, 1, 2, false>"][0] == 3
    assert not any(k.startswith("conv_fwd_strided_kernel<FpAr, 5, 2") for k in prof)
    assert all(n > 0 and ms > 0 and b > 0 for n, ms, b in prof.values())


def test_two_stream_overlap_gives_identical_results(orc):
    ps = synth.small_params(13, 6, 3, 2)
    ctx = gpu_ctx(ps)
    rng = np.random.default_rng(19)
    ct1 = dev(synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(3, 2)))
    ct2 = dev(synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(3, 2)))
    key = dev(synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2)))
    gs = [synth.galois_element(r, ps.logN) for r in range(1, 12)]
    rks = [dev(synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2))) for _ in gs]
    pt = dev(synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(len(gs),)))
    ref = [host(ctx.hmult_relin(ct1, ct2, key)), host(ctx.hrot(ct1, gs[2], key)),
           host(ctx.hrot_hoisted_mac(ct1[0].contiguous(), gs, rks, pt))]
    ctx.set_overlap(True)
    try:
        for _ in range(3):
            got = [host(ctx.hmult_relin(ct1, ct2, key)), host(ctx.hrot(ct1, gs[2], key)),
                   host(ctx.hrot_hoisted_mac(ct1[0].contiguous(), gs, rks, pt))]
            for a, b in zip(ref, got):
                assert np.array_equal(a, b)
    finally:
        ctx.set_overlap(False)


def test_caller_supplied_roots(orc):
    """A context created with the caller's own primitive 2N-th roots (odd powers of the minimal ones) transforms,
    rotates and switches keys with those roots, like the oracle given the same ones; a root of the wrong order is
    rejected on the host."""
    from paper_2310_16530_amd import binding
    ps = synth.small_params(13, 4, 2, 2)
    base = orc.Params(ps.logN, ps.L, ps.K, ps.dnum, ps.primes)
    rng = np.random.default_rng(515)
    psi = [pow(r, int(2 * rng.integers(1, ps.N) + 1), p) for r, p in zip(base.psi, ps.primes)]
    assert psi != base.psi
    P = orc.Params(ps.logN, ps.L, ps.K, ps.dnum, ps.primes, psi)
    ctx = binding.Context(ps.logN, ps.L, ps.K, ps.dnum, ps.primes, psi=psi)
    assert [ctx.psi(i) for i in range(ps.L + ps.K)] == psi
    x = synth.uniform_residues(rng, ps.primes, ps.N, lead=(2,))
    assert np.array_equal(host(ctx.ntt(dev(x))), orc.ntt_batch(x, P, 0))
    assert not np.array_equal(host(ctx.ntt(dev(x))), orc.ntt_batch(x, base, 0))
    assert np.array_equal(host(ctx.intt(dev(x))), orc.ntt_batch(x, P, 0, inverse=True))
    key = synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2))
    ct1 = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(2, 2))
    ct2 = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(2, 2))
    g = synth.galois_element(5, ps.logN)
    hm = host(ctx.hmult_relin(dev(ct1), dev(ct2), dev(key)))
    hr = host(ctx.hrot(dev(ct1), g, dev(key)))
    for b in range(2):
        assert np.array_equal(hm[b], orc.hmult_relin(ct1[b], ct2[b], key, P)), b
        assert np.array_equal(hr[b], orc.hrot(ct1[b], g, key, P)), b
    bad = list(psi)
    bad[1] = pow(psi[1], 2, ps.primes[1])       # order N, not 2N
    with pytest.raises(binding.CkksError):
        binding.Context(ps.logN, ps.L, ps.K, ps.dnum, ps.primes, psi=bad)
