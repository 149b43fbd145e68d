"""Parity of the level-aware entry points and of rescale against the CPU oracle, bit for bit (needs an MI355X).

Covers every level of several reduced shapes (full digits, a partial last digit, a single limb),
integer-arithmetic q-limbs as well as floating-point ones, a multiply-rescale chain, and the
benchmark shape N = 2^16, L = 24, dnum = 4 at a level whose last digit is partial.
"""
import ctypes

import numpy as np
import pytest

from paper_2310_16530_amd import synth

from test_gpu_parity import dev, gpu_ctx, host, make_keys, orc_params

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)


# (logN, L, K, dnum, q bits, p bits): 49-bit q-limbs use the FP64 arithmetic, 55-bit ones the integer one
RESCALE_SHAPES = [(12, 4, 2, 2, 49, 59), (13, 6, 3, 2, 49, 59), (12, 3, 1, 3, 35, 36), (14, 5, 0, 1, 49, 59),
                  (12, 4, 2, 2, 55, 59), (16, 3, 1, 3, 49, 59)]


@pytest.mark.parametrize("shape", RESCALE_SHAPES)
def test_rescale_parity_every_level(orc, shape):
    ps = synth.small_params(*shape)
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = np.random.default_rng(3000 + sum(shape))
    B = 3
    for ell in range(ps.L, 1, -1):
        _say("rescale", shape, "level", ell)
        ct = synth.uniform_residues(rng, ps.q_primes[:ell], ps.N, lead=(B, 2))
        ct[1, 0] = 0
        for i in range(ell):
            ct[2, 1, i, :] = ps.q_primes[i] - 1
        got = host(ctx.rescale(ell, dev(ct)))
        assert got.shape == (B, 2, ell - 1, ps.N)
        assert np.array_equal(got, orc.rescale(ct, P)), ell


LEVEL_SHAPES = [(12, 6, 2, 3, 49, 59), (13, 6, 3, 2, 49, 59), (12, 8, 8, 1, 49, 59), (12, 3, 1, 3, 35, 36),
                (12, 6, 3, 2, 55, 59), (12, 14, 7, 2, 49, 59), (12, 24, 12, 2, 49, 59), (12, 11, 11, 1, 55, 59),
                (12, 7, 3, 3, 49, 59), (12, 10, 4, 4, 55, 59)]   # last two: dnum does not divide L


@pytest.mark.parametrize("shape", LEVEL_SHAPES)
def test_keyswitch_hmult_hrot_parity_at_levels(orc, shape):
    ps = synth.small_params(*shape)
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = np.random.default_rng(4000 + sum(shape))
    s = synth.ternary_hamming(rng, ps.N, 64)
    s_hat = orc.secret_eval(s, P)
    s2_hat = orc.pointwise("mul", s_hat, s_hat, ps.primes)
    evk = make_keys(orc, ps, P, rng, s_hat, s2_hat)
    g = synth.galois_element(-3, ps.logN)
    rk = make_keys(orc, ps, P, rng, s_hat, orc.automorph_limbs(s_hat, P, 0, g, True))
    d_evk, d_rk = dev(evk), dev(rk)
    levels = sorted({ps.L, ps.L - 1, ps.alpha + 1, ps.alpha, max(ps.alpha - 1, 1), 1} & set(range(1, ps.L + 1)))
    B = 2
    for ell in levels:
        _say("levels", shape, "level", ell)
        q = ps.q_primes[:ell]
        d = synth.uniform_residues(rng, q, ps.N, lead=(B,))
        ks = host(ctx.keyswitch_at(ell, dev(d), d_evk))
        for b in range(B):
            assert np.array_equal(ks[b], orc.keyswitch_level(d[b], evk, P)), (ell, b)
        bound = orc.keyswitch_noise_bound(P, int(np.abs(s).sum()), level=ell)
        assert np.abs(orc.keyswitch_noise(d[0], ks[0], s_hat, s2_hat, P, level=ell)).max() <= bound
        ct1 = synth.uniform_residues(rng, q, ps.N, lead=(B, 2))
        ct2 = synth.uniform_residues(rng, q, ps.N, lead=(B, 2))
        hm = host(ctx.hmult_relin_at(ell, dev(ct1), dev(ct2), d_evk))
        hr = host(ctx.hrot_at(ell, dev(ct1), g, d_rk))
        for b in range(B):
            assert np.array_equal(hm[b], orc.hmult_relin_level(ct1[b], ct2[b], evk, P)), (ell, b)
            assert np.array_equal(hr[b], orc.hrot_level(ct1[b], g, rk, P)), (ell, b)
    # the full level through the level-aware entry equals the plain entry
    ct = dev(synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(B, 2)))
    assert np.array_equal(host(ctx.hrot_at(ps.L, ct, g, d_rk)), host(ctx.hrot(ct, g, d_rk)))


@pytest.mark.parametrize("shape,n_rot", [((12, 6, 2, 3, 49, 59), 3), ((13, 6, 3, 2, 49, 59), 11)])
def test_hoisted_mac_parity_at_levels(orc, shape, n_rot):
    ps = synth.small_params(*shape)
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = np.random.default_rng(5000 + sum(shape))
    rots = [1, 2, 3, 4, 5, 6, 7, 8, 16, -1, 32][:n_rot]
    gs = [synth.galois_element(r, ps.logN) for r in rots]
    rks = [synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2)) for _ in gs]
    d_rks = [dev(k) for k in rks]
    for ell in (ps.L - 1, ps.alpha + 1, 1):
        _say("hoisted", shape, "level", ell)
        q = ps.q_primes[:ell]
        ct = synth.uniform_residues(rng, q, ps.N, lead=(2,))
        pt = synth.uniform_residues(rng, q, ps.N, lead=(n_rot,))
        got = host(ctx.hrot_hoisted_mac_at(ell, dev(ct), gs, d_rks, dev(pt)))
        assert np.array_equal(got, orc.hrot_hoisted_mac_level(ct, gs, rks, pt, P)), ell


def test_multiply_rescale_chain(orc):
    """(ct1 * ct2 -> rescale) * ct3 -> rescale, every intermediate compared with the oracle."""
    ps = synth.small_params(13, 6, 2, 3)
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = np.random.default_rng(6000)
    evk = synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2))
    d_evk = dev(evk)
    L = ps.L
    ct1 = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(2,))
    ct2 = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(2,))
    ct3 = synth.uniform_residues(rng, ps.q_primes[:L - 1], ps.N, lead=(2,))
    g1 = ctx.hmult_relin_at(L, dev(ct1), dev(ct2), d_evk)
    w1 = orc.hmult_relin_level(ct1, ct2, evk, P)
    assert np.array_equal(host(g1), w1)
    g2 = ctx.rescale(L, g1)
    w2 = orc.rescale(w1, P)
    assert np.array_equal(host(g2), w2)
    g3 = ctx.hmult_relin_at(L - 1, g2, dev(ct3), d_evk)
    w3 = orc.hmult_relin_level(w2, ct3, evk, P)
    assert np.array_equal(host(g3), w3)
    g4 = host(ctx.rescale(L - 1, g3))
    assert np.array_equal(g4, orc.rescale(w3, P))


@pytest.mark.timeout(900)
def test_config2_shape_at_a_partial_level_full_size(orc):
    """N = 2^16, L = 24, K = 6, dnum = 4 at level 13 (digits of 6, 6 and 1 limbs), batch 8: HMult, rescale, HRot."""
    ps = synth.CFG2
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = synth.rng_for(2, 7)
    ell, B = 13, synth.CFG2_BATCH
    evk = synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2))
    q = ps.q_primes[:ell]
    ct1 = synth.uniform_residues(rng, q, ps.N, lead=(B, 2))
    ct2 = synth.uniform_residues(rng, q, ps.N, lead=(B, 2))
    d_evk = dev(evk)
    _say("cfg2 level 13: hmult")
    hm_d = ctx.hmult_relin_at(ell, dev(ct1), dev(ct2), d_evk)
    hm = host(hm_d)
    for b in range(B):
        assert np.array_equal(hm[b], orc.hmult_relin_level(ct1[b], ct2[b], evk, P)), b
    _say("cfg2 level 13: rescale")
    rs = host(ctx.rescale(ell, hm_d))
    assert np.array_equal(rs, orc.rescale(hm, P))
    _say("cfg2 level 13: hrot")
    g = synth.galois_element(5, ps.logN)
    hr = host(ctx.hrot_at(ell, dev(ct1), g, d_evk))
    for b in range(B):
        assert np.array_equal(hr[b], orc.hrot_level(ct1[b], g, evk, P)), b


def test_level_error_paths(orc):
    from paper_2310_16530_amd import binding
    import torch
    lib = binding.load()
    ps = synth.small_params(12, 4, 2, 2)
    ctx = gpu_ctx(ps)
    x = torch.zeros((1, 2, ps.L, ps.N), dtype=torch.int64, device="cuda:0")
    out = torch.empty_like(x)
    key = torch.zeros((ps.dnum, 2, ps.L + ps.K, ps.N), dtype=torch.int64, device="cuda:0")
    ws = ctx.workspace(binding.OP_HROT, 1)
    h, p, o, k, w = ctx.handle, x.data_ptr(), out.data_ptr(), key.data_ptr(), ws.data_ptr()
    for bad in (0, ps.L + 1):
        assert lib.ckks_keyswitch_at(h, bad, p, k, o, 1, w, ws.numel(), None) == binding.CKKS_EINVAL
        assert lib.ckks_hmult_relin_at(h, bad, p, p, k, o, 1, w, ws.numel(), None) == binding.CKKS_EINVAL
        assert lib.ckks_hrot_at(h, bad, p, 5, k, o, 1, w, ws.numel(), None) == binding.CKKS_EINVAL
        assert lib.ckks_rescale(h, bad, p, o, 1, w, ws.numel(), None) == binding.CKKS_EINVAL
    assert b"level" in lib.ckks_last_error(h)
    assert lib.ckks_rescale(h, 1, p, o, 1, w, ws.numel(), None) == binding.CKKS_EINVAL
    assert lib.ckks_rescale(h, 3, p, o, 1, w, 64, None) == binding.CKKS_ENOMEM
    assert lib.ckks_rescale(h, 3, p, None, 1, w, ws.numel(), None) == binding.CKKS_EINVAL
    n = ctypes.c_size_t()
    assert lib.ckks_workspace_bytes_at(h, binding.OP_KEYSWITCH, 9, 1, ctypes.byref(n)) == binding.CKKS_EINVAL
    sizes = []
    for ell in range(1, ps.L + 1):
        assert lib.ckks_workspace_bytes_at(h, binding.OP_HMULT_RELIN, ell, 2, ctypes.byref(n)) == 0
        sizes.append(n.value)
    assert sizes == sorted(sizes) and sizes[-1] == ctx.workspace_bytes(binding.OP_HMULT_RELIN, 2)
    torch.cuda.synchronize()


# ------------------------------------------------------------------ double hoisting
@pytest.mark.parametrize("shape,n_rot", [((12, 6, 2, 3, 49, 59), 3), ((13, 6, 3, 2, 49, 59), 11), ((12, 4, 2, 2, 55, 59), 5),
                                         ((12, 3, 1, 3, 35, 36), 37), ((12, 20, 1, 20, 49, 59), 4)])
def test_double_hoisted_mac_parity(orc, shape, n_rot):
    """Full level, a partial-digit level and a single limb; 37 rotations exceed one launch's chunk of 32."""
    ps = synth.small_params(*shape)
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = np.random.default_rng(7000 + sum(shape))
    gs = [synth.galois_element(r, ps.logN) for r in range(1, n_rot + 1)]
    rks = [synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2)) for _ in gs]
    d_rks = [dev(k) for k in rks]
    for ell in sorted({ps.L, max(ps.L - 1, 1), min(ps.alpha + 1, ps.L), 1}, reverse=True):
        _say("double hoisting", shape, "level", ell)
        basis = list(ps.q_primes[:ell]) + list(ps.p_primes)
        ct = synth.uniform_residues(rng, basis[:ell], ps.N, lead=(2,))
        pt = synth.uniform_residues(rng, basis, ps.N, lead=(n_rot,))
        want = orc.hrot_dh_mac_level(ct, gs, rks, pt, P)
        got = host(ctx.hrot_dh_mac(dev(ct), gs, d_rks, dev(pt), level=ell))
        assert np.array_equal(got, want), ell
        if ell == ps.L:
            assert np.array_equal(host(ctx.hrot_dh_mac(dev(ct), gs, d_rks, dev(pt))), want)
    # one rotation with the all-ones plaintext is that rotation of the singly hoisted path
    ct = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(2,))
    unit = np.ones((1, ps.L + ps.K, ps.N), dtype=np.uint64)
    one = host(ctx.hrot_dh_mac(dev(ct), gs[-1:], d_rks[-1:], dev(unit)))
    assert np.array_equal(one, host(ctx.hrot_hoisted_mac(dev(ct), gs[-1:], d_rks[-1:], dev(unit[:, :ps.L]))))


@pytest.mark.timeout(900)
def test_config3_double_hoisted_full_size(orc):
    """the shape of workload 3 (17 rotations, N = 2^16, L = 24, dnum = 4) through the double-hoisted call."""
    ps = synth.CFG3
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = synth.rng_for(3, 5)
    gs = [synth.galois_element(r, ps.logN) for r in synth.CFG3_ROTATIONS]
    rks = [synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2)) for _ in gs]
    ct = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(2,))
    pt = synth.uniform_residues(rng, ps.primes, ps.N, lead=(len(gs),))
    _say("cfg3 double hoisting: gpu")
    got = host(ctx.hrot_dh_mac(dev(ct), gs, [dev(k) for k in rks], dev(pt)))
    _say("cfg3 double hoisting: oracle")
    assert np.array_equal(got, orc.hrot_dh_mac_level(ct, gs, rks, pt, P))


# ------------------------------------------- ModDown merged with the following rescale
MERGED_SHAPES = [(12, 6, 2, 3, 49, 59), (13, 6, 3, 2, 49, 59), (12, 3, 1, 3, 35, 36), (12, 6, 3, 2, 55, 59),
                 (12, 8, 8, 1, 49, 59), (14, 4, 2, 2, 49, 59), (12, 10, 10, 1, 49, 59), (12, 18, 16, 2, 49, 59),
                 (12, 7, 3, 3, 49, 59)]


@pytest.mark.parametrize("shape", MERGED_SHAPES)
def test_hmult_relin_rescale_merged_parity_every_level(orc, shape):
    ps = synth.small_params(*shape)
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = np.random.default_rng(8000 + sum(shape))
    evk = synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2))
    d_evk = dev(evk)
    B = 2
    for ell in range(ps.L, 1, -1):
        _say("merged hmult", shape, "level", ell)
        q = ps.q_primes[:ell]
        ct1 = synth.uniform_residues(rng, q, ps.N, lead=(B, 2))
        ct2 = synth.uniform_residues(rng, q, ps.N, lead=(B, 2))
        got = host(ctx.hmult_relin_rescale_at(ell, dev(ct1), dev(ct2), d_evk))
        assert got.shape == (B, 2, ell - 1, ps.N)
        for b in range(B):
            assert np.array_equal(got[b], orc.hmult_relin_rescale_level(ct1[b], ct2[b], evk, P)), (ell, b)


@pytest.mark.parametrize("shape,n_rot", [((12, 6, 2, 3, 49, 59), 3), ((13, 6, 3, 2, 49, 59), 11), ((12, 4, 2, 2, 55, 59), 5)])
def test_double_hoisted_mac_rescale_merged_parity(orc, shape, n_rot):
    ps = synth.small_params(*shape)
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = np.random.default_rng(9000 + sum(shape))
    gs = [synth.galois_element(r, ps.logN) for r in range(1, n_rot + 1)]
    rks = [synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2)) for _ in gs]
    d_rks = [dev(k) for k in rks]
    for ell in sorted({ps.L, ps.L - 1, ps.alpha + 1, 2}, reverse=True):
        _say("merged double hoisting", shape, "level", ell)
        basis = list(ps.q_primes[:ell]) + list(ps.p_primes)
        ct = synth.uniform_residues(rng, basis[:ell], ps.N, lead=(2,))
        pt = synth.uniform_residues(rng, basis, ps.N, lead=(n_rot,))
        got = host(ctx.hrot_dh_mac_rescale_at(ell, dev(ct), gs, d_rks, dev(pt)))
        assert np.array_equal(got, orc.hrot_dh_mac_rescale_level(ct, gs, rks, pt, P)), ell


@pytest.mark.timeout(900)
def test_config2_shape_merged_rescale_full_size(orc):
    """N = 2^16, L = 24, K = 6, dnum = 4, batch 8: HMult+relin+rescale at levels 24 and 13; 17 double-hoisted
    rotations with rescale at level 24."""
    ps = synth.CFG2
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = synth.rng_for(2, 9)
    B = synth.CFG2_BATCH
    evk = synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2))
    d_evk = dev(evk)
    for ell, check in ((24, range(B)), (13, range(B))):
        q = ps.q_primes[:ell]
        ct1 = synth.uniform_residues(rng, q, ps.N, lead=(B, 2))
        ct2 = synth.uniform_residues(rng, q, ps.N, lead=(B, 2))
        _say("cfg2 merged hmult level", ell)
        got = host(ctx.hmult_relin_rescale_at(ell, dev(ct1), dev(ct2), d_evk))
        for b in check:
            assert np.array_equal(got[b], orc.hmult_relin_rescale_level(ct1[b], ct2[b], evk, P)), (ell, b)
    gs = [synth.galois_element(r, ps.logN) for r in synth.CFG3_ROTATIONS]
    rks = [np.roll(evk, i + 1, axis=-1) for i in range(len(gs))]
    ct = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(2,))
    pt = synth.uniform_residues(rng, ps.primes, ps.N, lead=(len(gs),))
    _say("cfg3 merged double hoisting")
    got = host(ctx.hrot_dh_mac_rescale_at(ps.L, dev(ct), gs, [dev(k) for k in rks], dev(pt)))
    assert np.array_equal(got, orc.hrot_dh_mac_rescale_level(ct, gs, rks, pt, P))


def test_merged_rescale_error_paths(orc):
    from paper_2310_16530_amd import binding
    import torch
    lib = binding.load()
    ps = synth.small_params(12, 4, 2, 2)
    ctx = gpu_ctx(ps)
    x = torch.zeros((1, 2, ps.L, ps.N), dtype=torch.int64, device="cuda:0")
    out = torch.empty_like(x)
    key = torch.zeros((ps.dnum, 2, ps.L + ps.K, ps.N), dtype=torch.int64, device="cuda:0")
    ws = ctx.workspace(binding.OP_HROT, 1)
    h, p, o, k, w = ctx.handle, x.data_ptr(), out.data_ptr(), key.data_ptr(), ws.data_ptr()
    for bad in (0, 1, ps.L + 1):
        assert lib.ckks_hmult_relin_rescale_at(h, bad, p, p, k, o, 1, w, ws.numel(), None) == binding.CKKS_EINVAL
    assert lib.ckks_hmult_relin_rescale_at(h, 3, p, p, k, o, 1, w, 128, None) == binding.CKKS_ENOMEM
    t_only = gpu_ctx(synth.small_params(12, 2, 0, 1))
    assert lib.ckks_hmult_relin_rescale_at(t_only.handle, 2, p, p, k, o, 1, w, ws.numel(), None) == binding.CKKS_EUNSUPPORTED
    torch.cuda.synchronize()


def test_two_stream_overlap_on_level_and_merged_entry_points(orc):
    """The optional two-stream execution must not change a single word of the newer entry points either."""
    ps = synth.small_params(13, 6, 3, 2)
    ctx = gpu_ctx(ps)
    rng = np.random.default_rng(29)
    ell = 5
    q = ps.q_primes[:ell]
    ct1 = dev(synth.uniform_residues(rng, q, ps.N, lead=(3, 2)))
    ct2 = dev(synth.uniform_residues(rng, q, ps.N, lead=(3, 2)))
    key = dev(synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2)))
    gs = [synth.galois_element(r, ps.logN) for r in range(1, 6)]
    rks = [dev(synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2))) for _ in gs]
    pt = dev(synth.uniform_residues(rng, list(q) + list(ps.p_primes), ps.N, lead=(len(gs),)))
    one = ct1[0].contiguous()

    def run():
        return [host(ctx.hmult_relin_at(ell, ct1, ct2, key)), host(ctx.hrot_at(ell, ct1, gs[1], key)),
                host(ctx.rescale(ell, ct1)), host(ctx.hmult_relin_rescale_at(ell, ct1, ct2, key)),
                host(ctx.hrot_hoisted_mac_at(ell, one, gs, rks, pt[:, :ell].contiguous())),
                host(ctx.hrot_dh_mac(one, gs, rks, pt, level=ell)),
                host(ctx.hrot_dh_mac_rescale_at(ell, one, gs, rks, pt))]

    ref = run()
    ctx.set_overlap(True)
    try:
        for _ in range(3):
            for a, b in zip(ref, run()):
                assert np.array_equal(a, b)
    finally:
        ctx.set_overlap(False)


# ------------------------------------------------ baby-step giant-step linear transform
@pytest.mark.parametrize("shape,n1,n2", [((12, 6, 2, 3, 49, 59), 3, 2), ((13, 6, 3, 2, 49, 59), 4, 3),
                                         ((12, 4, 2, 2, 55, 59), 2, 2), ((12, 3, 1, 3, 35, 36), 9, 18)])
def test_bsgs_linear_transform_parity(orc, shape, n1, n2):
    """Includes identity rotations (Galois element 1) and more giant steps than one launch takes (18 > 16)."""
    ps = synth.small_params(*shape)
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = np.random.default_rng(11000 + sum(shape))
    baby = [synth.galois_element(r, ps.logN) for r in range(n1)]
    giant = [synth.galois_element(r * n1, ps.logN) for r in range(n2)]
    assert baby[0] == 1 and giant[0] == 1
    baby_rks = [synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2)) for _ in baby]
    giant_rks = [synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2)) for _ in giant]
    d_baby, d_giant = [dev(k) for k in baby_rks], [dev(k) for k in giant_rks]
    for ell in sorted({ps.L, max(ps.alpha + 1, 2) if ps.L > 2 else ps.L, 1}, reverse=True):
        _say("bsgs", shape, "level", ell)
        basis = list(ps.q_primes[:ell]) + list(ps.p_primes)
        ct = synth.uniform_residues(rng, basis[:ell], ps.N, lead=(2,))
        pt = synth.uniform_residues(rng, basis, ps.N, lead=(n2, n1))
        want = orc.lintrans_bsgs_level(ct, baby, baby_rks, giant, giant_rks, pt, P)
        got = host(ctx.lintrans_bsgs_at(ell, dev(ct), baby, d_baby, giant, d_giant, dev(pt)))
        assert np.array_equal(got, want), ell


@pytest.mark.timeout(600)
def test_bsgs_with_encoded_diagonals_is_a_matrix_vector_product(orc):
    """Real diagonals instead of random residues: a band matrix with 32 non-zero (generalised) diagonals on the 2048
    slots of N = 4096, encoded by the oracle's canonical embedding, true rotation keys, a fresh encryption of z.
    The library's baby-step giant-step call equals the oracle's word for word, and what it returns decrypts and
    decodes to M z."""
    ps = synth.small_params(12, 4, 2, 2, 49, 59)
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = np.random.default_rng(4242)
    N, n, ell = ps.N, ps.N // 2, ps.L
    n1, n2 = 8, 4
    scale = scale_pt = float(1 << 30)
    s = synth.ternary_hamming(rng, N, 64)
    s_hat = orc.secret_eval(s, P)
    diags = (rng.uniform(-1, 1, (n1 * n2, n)) + 1j * rng.uniform(-1, 1, (n1 * n2, n))) / np.sqrt(2)
    M = np.zeros((n, n), dtype=np.complex128)
    j = np.arange(n)
    for d in range(n1 * n2):
        M[j, (j + d) % n] = diags[d]
    z = (rng.uniform(-1, 1, n) + 1j * rng.uniform(-1, 1, n)) / np.sqrt(2)
    baby = [synth.galois_element(b, ps.logN) for b in range(n1)]
    giant = [synth.galois_element(g * n1, ps.logN) for g in range(n2)]
    _say("encoded diagonals: keys")
    baby_rks = [make_keys(orc, ps, P, rng, s_hat, orc.automorph_limbs(s_hat, P, 0, g, True)) for g in baby]
    giant_rks = [make_keys(orc, ps, P, rng, s_hat, orc.automorph_limbs(s_hat, P, 0, g, True)) for g in giant]
    q = list(ps.q_primes)
    sq = s_hat[:ell]
    _say("encoded diagonals: encode")
    m_hat = orc.encode_limbs(z, scale, P, q, P.psi[:ell])
    a = synth.uniform_residues(rng, q, N)
    e_hat = orc.ntt_batch(orc.lift_signed(synth.gaussian_error(rng, (N,)), q), P, 0)
    b = orc.pointwise("add", orc.pointwise("sub", m_hat, orc.pointwise("mul", a, sq, q), q), e_hat, q)
    ct = np.stack([b, a])
    pt = orc.bsgs_diagonal_plaintexts(M, n1, n2, scale_pt, P, ell)
    _say("encoded diagonals: gpu")
    got = host(ctx.lintrans_bsgs_at(ell, dev(ct), baby, [dev(k) for k in baby_rks], giant, [dev(k) for k in giant_rks], dev(pt)))
    _say("encoded diagonals: oracle")
    assert np.array_equal(got, orc.lintrans_bsgs_level(ct, baby, baby_rks, giant, giant_rks, pt, P))
    dec = orc.pointwise("add", got[0], orc.pointwise("mul", got[1], sq, q), q)
    slots = orc.decode(np.array(orc.crt_centred(dec, P, ell), dtype=np.float64), scale * scale_pt, ps.logN)
    # worst-case slot error, as in the CPU pin of the oracle: a coefficient error c moves a slot by at most N * c; every
    # slot sums 32 products of values of modulus <= 1 (message rounding 1/2 and encryption error <= 19 per coefficient,
    # diagonal rounding 1/2), plus the key-switch noise of the call
    h = int(np.abs(s).sum())
    l1 = [sum(int(np.abs(orc.centred_small(pt[g, bb], P, ell)).sum()) for bb in range(n1)) for g in range(n2)]
    noise = sum(orc.dh_mac_noise_bound(P, h, t, level=ell) for t in l1) + n2 * orc.keyswitch_noise_bound(P, h, level=ell)
    tol = n1 * n2 * (N / 2 + 19 * N) / scale + n1 * n2 * (N / 2) / scale_pt + N * noise / (scale * scale_pt)
    assert np.abs(slots - M @ z).max() <= tol < 0.01


@pytest.mark.timeout(900)
def test_bsgs_linear_transform_full_size(orc):
    """N = 2^16, L = 24, K = 6, dnum = 4: 8 baby steps x 4 giant steps (32 diagonals) at level 24."""
    ps = synth.CFG2
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = synth.rng_for(4, 11)
    n1, n2 = 8, 4
    baby = [synth.galois_element(r, ps.logN) for r in range(n1)]
    giant = [synth.galois_element(r * n1, ps.logN) for r in range(n2)]
    base = synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2))
    baby_rks = [np.roll(base, i + 1, axis=-1) for i in range(n1)]
    giant_rks = [np.roll(base, 100 + i, axis=-1) for i in range(n2)]
    ct = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(2,))
    pt = synth.uniform_residues(rng, ps.primes, ps.N, lead=(n2, n1))
    _say("bsgs full size: gpu")
    got = host(ctx.lintrans_bsgs_at(ps.L, dev(ct), baby, [dev(k) for k in baby_rks], giant, [dev(k) for k in giant_rks],
                                    dev(pt)))
    _say("bsgs full size: oracle")
    assert np.array_equal(got, orc.lintrans_bsgs_level(ct, baby, baby_rks, giant, giant_rks, pt, P))


@pytest.mark.parametrize("overlap", [False, True])
def test_entry_points_can_be_captured_in_a_graph_and_replayed(orc, overlap):
    """The library allocates nothing and issues only kernel launches, so a caller may capture its calls in a
    HIP graph.  Every replay (with eager work and synchronisations in between) must reproduce the eager result.
    With the library's second stream on, its fork and join by events are captured with the rest."""
    import torch
    from paper_2310_16530_amd import binding
    ps = synth.small_params(13, 6, 3, 2)
    ctx = binding.Context(ps.logN, ps.L, ps.K, ps.dnum, ps.primes)
    rng = np.random.default_rng(31)
    ell = 5
    q = ps.q_primes[:ell]
    ct1 = dev(synth.uniform_residues(rng, q, ps.N, lead=(2, 2)))
    ct2 = dev(synth.uniform_residues(rng, q, ps.N, lead=(2, 2)))
    key = dev(synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2)))
    gs = [synth.galois_element(r, ps.logN) for r in range(1, 4)]
    rks = [dev(synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2))) for _ in gs]
    pt = dev(synth.uniform_residues(rng, list(q) + list(ps.p_primes), ps.N, lead=(len(gs),)))
    one = ct1[0].contiguous()
    o_mult, o_low, o_rot = torch.empty_like(ct1), torch.empty_like(ct1[:, :, :ell - 1]).contiguous(), torch.empty_like(ct1)
    o_dh = torch.empty_like(one)
    # size the shared workspace for the largest call before capturing (no allocation may happen inside)
    for _ in range(2):
        ctx.hmult_relin_at(ell, ct1, ct2, key, o_mult)
        ctx.rescale(ell, o_mult, o_low)
        ctx.hrot_at(ell, ct1, gs[0], key, o_rot)
        ctx.hrot_dh_mac(one, gs, rks, pt, o_dh, level=ell)
    torch.cuda.synchronize()
    want = [host(o_mult).copy(), host(o_low).copy(), host(o_rot).copy(), host(o_dh).copy()]
    ctx.set_overlap(overlap)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ctx.hmult_relin_at(ell, ct1, ct2, key, o_mult)
        ctx.rescale(ell, o_mult, o_low)
        ctx.hrot_at(ell, ct1, gs[0], key, o_rot)
        ctx.hrot_dh_mac(one, gs, rks, pt, o_dh, level=ell)
    for rep in range(3):
        for o in (o_mult, o_low, o_rot, o_dh):
            o.fill_(rep + 7)                      # eager work between replays; also destroys the previous result
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(want, (o_mult, o_low, o_rot, o_dh)):
            assert np.array_equal(a, host(b)), rep


def test_hrot_multi_parity(orc):
    """19 ciphertexts, each rotated by its own element with its own key (two launches: 16 + 3 instances)."""
    ps = synth.small_params(12, 6, 2, 3)
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = np.random.default_rng(41)
    B = 19
    gs = [synth.galois_element(r, ps.logN) for r in (0, 1, -1, 2, 3, 5, 8, 13, 21, 34, 55, 89, 144, 233, 377, 610, -2, -3, 7)]
    rks = [synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2)) for _ in gs]
    d_rks = [dev(k) for k in rks]
    for ell in (ps.L, 3):
        ct = synth.uniform_residues(rng, ps.q_primes[:ell], ps.N, lead=(B, 2))
        got = host(ctx.hrot_multi_at(ell, dev(ct), gs, d_rks))
        for b in range(B):
            assert np.array_equal(got[b], orc.hrot_level(ct[b], gs[b], rks[b], P)), (ell, b)


def test_large_batches(orc):
    """Batches well above the benchmark's 8 (37 and 300 ciphertexts): every entry checked for the small one,
    sampled entries for the large one."""
    ps = synth.small_params(12, 4, 2, 2)
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = np.random.default_rng(53)
    key = synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2))
    d_key = dev(key)
    g = synth.galois_element(9, ps.logN)
    for B, check in ((37, range(37)), (300, (0, 1, 149, 298, 299))):
        _say("batch", B)
        ct1 = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(B, 2))
        ct2 = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(B, 2))
        hm = host(ctx.hmult_relin(dev(ct1), dev(ct2), d_key))
        hr = host(ctx.hrot(dev(ct1), g, d_key))
        rs = host(ctx.rescale(ps.L, dev(ct1)))
        mr = host(ctx.hmult_relin_rescale_at(ps.L, dev(ct1), dev(ct2), d_key))
        for b in check:
            assert np.array_equal(hm[b], orc.hmult_relin(ct1[b], ct2[b], key, P)), (B, b)
            assert np.array_equal(hr[b], orc.hrot(ct1[b], g, key, P)), (B, b)
            assert np.array_equal(rs[b], orc.rescale(ct1[b], P)), (B, b)
            assert np.array_equal(mr[b], orc.hmult_relin_rescale_level(ct1[b], ct2[b], key, P)), (B, b)


@pytest.mark.parametrize("shape", [(12, 6, 2, 3, 49, 59), (13, 6, 3, 2, 49, 59), (12, 4, 2, 2, 55, 59)])
def test_quadratic_activation_composed_from_library_calls(orc, shape):
    """w2 * x^2 + w1 * x on a batch of ciphertexts (the shape of a polynomial activation): square with merged
    rescale, two plaintext products, two rescales, a limb drop and a sum, every step through the library and
    mirrored call by call with the oracle."""
    from paper_2310_16530_amd import binding
    ps = synth.small_params(*shape)
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = np.random.default_rng(9500 + sum(shape))
    evk = synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2))
    d_evk = dev(evk)
    B, ell = 3, ps.L
    q = ps.q_primes
    x = synth.uniform_residues(rng, q[:ell], ps.N, lead=(B, 2))
    w1 = synth.uniform_residues(rng, q[:ell], ps.N, lead=(1,))
    w2 = synth.uniform_residues(rng, q[:ell - 1], ps.N, lead=(1,))
    dx = dev(x)
    # GPU
    sq = ctx.hmult_relin_rescale_at(ell, dx, dx, d_evk)                               # level ell - 1
    a = ctx.rescale(ell - 1, ctx.pointwise(binding.PW_MUL, sq, dev(w2)))               # level ell - 2
    b = ctx.rescale(ell, ctx.pointwise(binding.PW_MUL, dx, dev(w1)))                   # level ell - 1
    b = b[:, :, :ell - 2].contiguous()                                                 # drop a limb
    got = host(ctx.pointwise(binding.PW_ADD, a, b))
    # oracle
    for i in range(B):
        o_sq = orc.hmult_relin_rescale_level(x[i], x[i], evk, P)
        o_a = orc.rescale(np.stack([orc.pointwise("mul", o_sq[t], w2[0], q[:ell - 1]) for t in range(2)]), P)
        o_b = orc.rescale(np.stack([orc.pointwise("mul", x[i, t], w1[0], q[:ell]) for t in range(2)]), P)
        want = np.stack([orc.pointwise("add", o_a[t], o_b[t, :ell - 2], q[:ell - 2]) for t in range(2)])
        assert np.array_equal(got[i], want), i


@pytest.mark.parametrize("shape", [(12, 6, 2, 3, 49, 59), (13, 6, 3, 2, 49, 59)])
def test_factorised_transform_chain(orc, shape):
    """Three baby-step giant-step stages with growing rotation strides and a rescale after each one (the shape
    of a factorised slot transform): stage s works at level L - s on ready plaintext diagonals; every stage and
    every rescale goes through the library and is mirrored call by call with the oracle."""
    ps = synth.small_params(*shape)
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    rng = np.random.default_rng(12000 + sum(shape))
    stages = [(4, 2), (2, 2), (3, 1)]           # (baby steps, giant steps)
    keys, d_keys = {}, {}

    def key_for(g):                              # one key per Galois element, shared by the stages
        if g not in keys:
            keys[g] = synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2))
            d_keys[g] = dev(keys[g])
        return g

    ct = synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(2,))
    d_ct, o_ct = dev(ct), ct
    stride = 1
    for s, (n1, n2) in enumerate(stages):
        ell = ps.L - s
        _say("transform chain", shape, "stage", s, "level", ell)
        baby = [key_for(synth.galois_element(b * stride, ps.logN)) for b in range(n1)]
        giant = [key_for(synth.galois_element(g * n1 * stride, ps.logN)) for g in range(n2)]
        basis = list(ps.q_primes[:ell]) + list(ps.p_primes)
        pt = synth.uniform_residues(rng, basis, ps.N, lead=(n2, n1))
        d_ct = ctx.rescale(ell, ctx.lintrans_bsgs_at(ell, d_ct, baby, [d_keys[g] for g in baby], giant,
                                                     [d_keys[g] for g in giant], dev(pt))[None])[0]
        o_ct = orc.rescale(orc.lintrans_bsgs_level(o_ct, baby, [keys[g] for g in baby], giant, [keys[g] for g in giant],
                                                   pt, P), P)
        assert np.array_equal(host(d_ct), o_ct), s
        stride *= n1 * n2


def test_operands_and_workspace_beyond_4_gib(orc):
    """1100 ciphertexts at N = 2^16: every operand, result and workspace part is larger than 4 GiB, so word offsets
    that were computed in 32 bits would wrap.  Inputs are drawn on the device; first, middle and last entries are
    compared with the oracle, with and without the library's second stream."""
    import torch
    ps = synth.small_params(16, 4, 2, 2)
    ctx, P = gpu_ctx(ps), orc_params(orc, ps)
    B, N, L = 1100, ps.N, ps.L
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)

    def draw():
        x = torch.empty((B, 2, L, N), dtype=torch.int64, device="cuda")
        for i, q in enumerate(ps.q_primes):
            x[:, :, i, :] = torch.randint(0, q, (B, 2, N), generator=gen, device="cuda", dtype=torch.int64)
        return x

    ct1, ct2 = draw(), draw()
    assert ct1.numel() * 8 > 1 << 32
    key = synth.uniform_residues(np.random.default_rng(3), ps.primes, N, lead=(ps.dnum, 2))
    d_key = dev(key)
    g = synth.galois_element(11, ps.logN)
    try:
        for overlap in (False, True):
            _say("1100 ciphertexts, second stream", overlap)
            ctx.set_overlap(overlap)
            hm = ctx.hmult_relin(ct1, ct2, d_key)
            hr = ctx.hrot(ct1, g, d_key)
            ks = ctx.keyswitch_at(L, ct1[:, 0].contiguous(), d_key)
            rs = ctx.rescale(L, ct1)
            for b in (0, 549, 1099):
                a1, a2 = host(ct1[b]), host(ct2[b])
                assert np.array_equal(host(hm[b]), orc.hmult_relin(a1, a2, key, P)), ("hmult", b)
                assert np.array_equal(host(hr[b]), orc.hrot(a1, g, key, P)), ("hrot", b)
                assert np.array_equal(host(ks[b]), orc.keyswitch_level(a1[0], key, P)), ("keyswitch", b)
                assert np.array_equal(host(rs[b]), orc.rescale(a1[None], P)[0]), ("rescale", b)
            del hm, hr, ks, rs
    finally:
        ctx.set_overlap(False)
        ctx._ws.clear()          # the cached context of the test module should not keep tens of GiB of workspace
        torch.cuda.empty_cache()


@pytest.mark.parametrize("overlap", [False, True])
def test_calls_on_two_caller_streams_at_once(orc, overlap):
    """One context used under two torch streams: the binding keeps one workspace per stream, so an HMult batch and
    a rotation batch may run at the same time (the library's own second stream, when on, is shared by both)."""
    import torch
    from paper_2310_16530_amd import binding
    ps = synth.small_params(14, 6, 3, 2)
    ctx = binding.Context(ps.logN, ps.L, ps.K, ps.dnum, ps.primes)
    rng = np.random.default_rng(61)
    B = 6
    ct1 = dev(synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(B, 2)))
    ct2 = dev(synth.uniform_residues(rng, ps.q_primes, ps.N, lead=(B, 2)))
    evk = dev(synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2)))
    rk = dev(synth.uniform_residues(rng, ps.primes, ps.N, lead=(ps.dnum, 2)))
    g = synth.galois_element(3, ps.logN)
    want1, want2 = host(ctx.hmult_relin(ct1, ct2, evk)).copy(), host(ctx.hrot(ct1, g, rk)).copy()
    P = orc_params(orc, ps)
    assert np.array_equal(want1[B - 1], orc.hmult_relin(host(ct1[B - 1]), host(ct2[B - 1]), host(evk), P))
    ctx.set_overlap(overlap)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    o1, o2 = torch.empty_like(ct1), torch.empty_like(ct1)
    for rep in range(5):
        o1.fill_(1)
        o2.fill_(2)
        torch.cuda.synchronize()
        with torch.cuda.stream(s1):
            ctx.hmult_relin(ct1, ct2, evk, o1)
        with torch.cuda.stream(s2):
            ctx.hrot(ct1, g, rk, o2)
        torch.cuda.synchronize()
        assert np.array_equal(host(o1), want1), ("hmult", rep)
        assert np.array_equal(host(o2), want2), ("hrot", rep)
