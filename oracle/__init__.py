"""ctypes front end of the CPU oracle (oracle/ckks_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package; the HIP library and its binding never do.  Besides thin wrappers of the C
functions it holds the harness-side steps the key-switch path itself does not
export: lifting a small signed polynomial to RNS limbs, switching-key
generation (from random draws handed in by the caller) and the
decrypt-and-bound noise check; and the canonical-embedding encoding of slot vectors and of the
diagonals of a matrix, which turns the baby-step giant-step call into a matrix-vector product on the
slots (the shape of the CoeffToSlot / SlotToCoeff stages behind the paper's Table 1 "Boot" rows).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ckks_oracle.c")
_LIB = os.path.join(_HERE, "libckks_oracle.so")

_u64 = ctypes.c_uint64
_u32 = ctypes.c_uint32
_p = ctypes.c_void_p


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, OpenMP over limbs)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        override = os.environ.get("CKKS_ORACLE_LIB")  # the mutation tests point this at a sabotaged build
        if override:
            _lib = ctypes.CDLL(override)
        else:
            build()
            _lib = ctypes.CDLL(_LIB)
        for name in ("orc_mulmod", "orc_addmod", "orc_submod", "orc_powmod"):
            f = getattr(_lib, name)
            f.restype, f.argtypes = _u64, [_u64, _u64, _u64]
        _lib.orc_invmod.restype, _lib.orc_invmod.argtypes = _u64, [_u64, _u64]
        _lib.orc_min_psi.restype, _lib.orc_min_psi.argtypes = _u64, [_u64, _u32]
        _lib.orc_ntt_def_at.restype = _u64
        _lib.orc_ntt_def_at.argtypes = [_p, _u32, _u64, _u64, _u32]
    return _lib


def threads() -> int:
    """OpenMP threads the limb loops run on."""
    return int(lib().orc_threads())


def set_threads(n: int) -> None:
    """Pin the number of OpenMP threads (timing only; results do not depend on it)."""
    lib().orc_set_threads(ctypes.c_int(n))


def _ptr(a: np.ndarray):
    assert a.flags["C_CONTIGUOUS"], "oracle buffers must be contiguous"
    return ctypes.c_void_p(a.ctypes.data)


def _arr_u64(v: Sequence[int]) -> np.ndarray:
    return np.ascontiguousarray(np.array([int(x) for x in v], dtype=np.uint64))


# ------------------------------------------------------------------ parameters
class Params:
    """Primes (q's then p's) and the minimal primitive 2N-th roots the oracle derives itself."""

    def __init__(self, logN: int, L: int, K: int, dnum: int, primes: Sequence[int],
                 psi: Optional[Sequence[int]] = None):
        assert len(primes) == L + K
        # digits of alpha = ceil(L/dnum) limbs, the last one shorter when dnum does not divide L; dnum must be
        # the number of digits this gives
        assert dnum >= 1 and -(-L // -(-L // dnum)) == dnum
        self.logN, self.L, self.K, self.dnum = logN, L, K, dnum
        self.N = 1 << logN
        self.alpha = -(-L // dnum)
        self.even = L % dnum == 0   # the full-level C functions are written for digits of equal size
        self.primes = [int(p) for p in primes]
        self.psi = [int(x) for x in psi] if psi is not None else [min_psi(p, logN) for p in self.primes]
        self._primes = _arr_u64(self.primes)
        self._psi = _arr_u64(self.psi)

    @classmethod
    def from_set(cls, ps) -> "Params":
        return cls(ps.logN, ps.L, ps.K, ps.dnum, ps.primes)

    def _tail(self):
        return (_u32(self.logN), _u32(self.L), _u32(self.K), _u32(self.dnum), _ptr(self._primes), _ptr(self._psi))


# --------------------------------------------------------------------- scalars
def mulmod(a, b, m):
    return int(lib().orc_mulmod(int(a), int(b), int(m)))


def powmod(a, e, m):
    return int(lib().orc_powmod(int(a), int(e), int(m)))


def invmod(a, m):
    return int(lib().orc_invmod(int(a), int(m)))


def min_psi(m: int, logN: int) -> int:
    return int(lib().orc_min_psi(int(m), int(logN)))


# ------------------------------------------------------------------ transforms
def ntt_def(x: np.ndarray, logN: int, m: int, psi: int) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.uint64)
    out = np.empty_like(x)
    lib().orc_ntt_def(_ptr(x), _ptr(out), _u32(logN), _u64(m), _u64(psi))
    return out


def ntt_def_at(x: np.ndarray, logN: int, m: int, psi: int, j: int) -> int:
    x = np.ascontiguousarray(x, dtype=np.uint64)
    return int(lib().orc_ntt_def_at(_ptr(x), logN, m, psi, j))


def ntt(x: np.ndarray, logN: int, m: int, psi: int) -> np.ndarray:
    out = np.array(x, dtype=np.uint64, copy=True, order="C")
    lib().orc_ntt(_ptr(out), _u32(logN), _u64(m), _u64(psi))
    return out


def intt(x: np.ndarray, logN: int, m: int, psi: int) -> np.ndarray:
    out = np.array(x, dtype=np.uint64, copy=True, order="C")
    lib().orc_intt(_ptr(out), _u32(logN), _u64(m), _u64(psi))
    return out


def ntt_batch(x: np.ndarray, P: Params, prime_first: int, inverse: bool = False) -> np.ndarray:
    """x: [batch][n_limbs][N] (or [n_limbs][N]); limb l uses prime prime_first + l."""
    out = np.array(x, dtype=np.uint64, copy=True, order="C")
    n_limbs = out.shape[-2]
    batch = int(np.prod(out.shape[:-2])) if out.ndim > 2 else 1
    pr = _arr_u64(P.primes[prime_first:prime_first + n_limbs])
    ps = _arr_u64(P.psi[prime_first:prime_first + n_limbs])
    lib().orc_ntt_batch(_ptr(out), _u32(P.logN), _u32(n_limbs), _u32(batch), _ptr(pr), _ptr(ps),
                        ctypes.c_int(1 if inverse else 0))
    return out


# ------------------------------------------------------------- base conversion
def conv(x: np.ndarray, src: Sequence[int], b: int) -> np.ndarray:
    """x: [len(src)][N] -> [N] residues modulo b (uncorrected fast base conversion)."""
    x = np.ascontiguousarray(x, dtype=np.uint64)
    n = x.shape[-1]
    out = np.empty(n, dtype=np.uint64)
    s = _arr_u64(src)
    lib().orc_conv(_ptr(x), ctypes.c_size_t(n), ctypes.c_size_t(n), _ptr(s), _u32(len(src)), _u64(b), _ptr(out))
    return out


def modup(x: np.ndarray, P: Params) -> np.ndarray:
    """[L][N] coefficient form -> [dnum][L+K][N] coefficient form."""
    x = np.ascontiguousarray(x, dtype=np.uint64)
    if not P.even:
        return modup_level(x, P)
    out = np.empty((P.dnum, P.L + P.K, P.N), dtype=np.uint64)
    lib().orc_modup(_ptr(x), _ptr(out), _u32(P.logN), _u32(P.L), _u32(P.K), _u32(P.dnum), _ptr(P._primes))
    return out


def moddown(x: np.ndarray, P: Params) -> np.ndarray:
    """[L+K][N] coefficient form -> [L][N] coefficient form."""
    x = np.ascontiguousarray(x, dtype=np.uint64)
    out = np.empty((P.L, P.N), dtype=np.uint64)
    lib().orc_moddown(_ptr(x), _ptr(out), _u32(P.logN), _u32(P.L), _u32(P.K), _ptr(P._primes))
    return out


# ---------------------------------------------------------------- automorphism
def automorph_coeff(x: np.ndarray, logN: int, m: int, g: int) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.uint64)
    out = np.empty_like(x)
    lib().orc_automorph_coeff(_ptr(x), _ptr(out), _u32(logN), _u64(m), _u32(g))
    return out


def automorph_eval(x: np.ndarray, logN: int, g: int) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.uint64)
    out = np.empty_like(x)
    lib().orc_automorph_eval(_ptr(x), _ptr(out), _u32(logN), _u32(g))
    return out


def automorph_limbs(x: np.ndarray, P: Params, prime_first: int, g: int, eval_domain: bool) -> np.ndarray:
    """Apply sigma_g to every limb of [..., n_limbs, N]; limb l uses prime prime_first + l."""
    x = np.ascontiguousarray(x, dtype=np.uint64)
    flat = x.reshape(-1, x.shape[-2], x.shape[-1])
    out = np.empty_like(flat)
    for b in range(flat.shape[0]):
        for l in range(flat.shape[1]):
            if eval_domain:
                out[b, l] = automorph_eval(flat[b, l], P.logN, g)
            else:
                out[b, l] = automorph_coeff(flat[b, l], P.logN, P.primes[prime_first + l], g)
    return out.reshape(x.shape)


# ---------------------------------------------------------------- compositions
def keyswitch(d: np.ndarray, key: np.ndarray, P: Params) -> np.ndarray:
    """d [L][N] eval, key [dnum][2][L+K][N] eval -> [2][L][N] eval."""
    d = np.ascontiguousarray(d, dtype=np.uint64)
    key = np.ascontiguousarray(key, dtype=np.uint64)
    assert d.shape == (P.L, P.N) and key.shape == (P.dnum, 2, P.L + P.K, P.N)
    if not P.even:
        return keyswitch_level(d, key, P)
    out = np.empty((2, P.L, P.N), dtype=np.uint64)
    lib().orc_keyswitch(_ptr(d), _ptr(key), _ptr(out), *P._tail())
    return out


def hmult_relin(ct1: np.ndarray, ct2: np.ndarray, evk: np.ndarray, P: Params) -> np.ndarray:
    ct1 = np.ascontiguousarray(ct1, dtype=np.uint64)
    ct2 = np.ascontiguousarray(ct2, dtype=np.uint64)
    evk = np.ascontiguousarray(evk, dtype=np.uint64)
    assert ct1.shape == ct2.shape == (2, P.L, P.N) and evk.shape == (P.dnum, 2, P.L + P.K, P.N)
    if not P.even:
        return hmult_relin_level(ct1, ct2, evk, P)
    out = np.empty((2, P.L, P.N), dtype=np.uint64)
    lib().orc_hmult_relin(_ptr(ct1), _ptr(ct2), _ptr(evk), _ptr(out), *P._tail())
    return out


def hrot(ct: np.ndarray, g: int, rk: np.ndarray, P: Params) -> np.ndarray:
    ct = np.ascontiguousarray(ct, dtype=np.uint64)
    rk = np.ascontiguousarray(rk, dtype=np.uint64)
    assert ct.shape == (2, P.L, P.N) and rk.shape == (P.dnum, 2, P.L + P.K, P.N)
    if not P.even:
        return hrot_level(ct, g, rk, P)
    out = np.empty((2, P.L, P.N), dtype=np.uint64)
    lib().orc_hrot(_ptr(ct), _u32(g), _ptr(rk), _ptr(out), *P._tail())
    return out


def hrot_hoisted_mac(ct: np.ndarray, galois: Sequence[int], rks: Sequence[np.ndarray], pt: np.ndarray,
                     P: Params, want_per_rotation: bool = False):
    """ct [2][L][N]; rks: one [dnum][2][L+K][N] key per rotation; pt [n_rot][L][N] -> [2][L][N]."""
    ct = np.ascontiguousarray(ct, dtype=np.uint64)
    pt = np.ascontiguousarray(pt, dtype=np.uint64)
    n_rot = len(galois)
    assert len(rks) == n_rot and pt.shape == (n_rot, P.L, P.N)
    if not P.even and not want_per_rotation:
        return hrot_hoisted_mac_level(ct, galois, rks, pt, P)
    assert P.even, "per-rotation outputs are provided for digits of equal size only"
    rks = [np.ascontiguousarray(k, dtype=np.uint64) for k in rks]
    ptrs = (ctypes.c_void_p * n_rot)(*[k.ctypes.data for k in rks])
    g = np.ascontiguousarray(np.array(galois, dtype=np.uint32))
    out = np.empty((2, P.L, P.N), dtype=np.uint64)
    per = np.empty((n_rot, 2, P.L, P.N), dtype=np.uint64) if want_per_rotation else None
    lib().orc_hrot_hoisted_mac(_ptr(ct), _u32(n_rot), _ptr(g), ptrs, _ptr(pt), _ptr(out),
                               _ptr(per) if per is not None else None, *P._tail())
    return (out, per) if want_per_rotation else out


# ----------------------------------------------------- levels below L, rescale
def _level_tail(P: Params, level: int):
    assert 1 <= level <= P.L
    return (_u32(level),) + P._tail()


def rescale(x: np.ndarray, P: Params) -> np.ndarray:
    """[..., ell, N] eval -> [..., ell-1, N] eval: every polynomial divided by q_{ell-1} (floor type)."""
    x = np.ascontiguousarray(x, dtype=np.uint64)
    ell = x.shape[-2]
    assert 2 <= ell <= P.L and x.shape[-1] == P.N
    flat = x.reshape(-1, ell, P.N)
    out = np.empty((flat.shape[0], ell - 1, P.N), dtype=np.uint64)
    for b in range(flat.shape[0]):
        lib().orc_rescale(_ptr(flat[b]), _ptr(out[b]), _u32(P.logN), _u32(ell), _ptr(P._primes), _ptr(P._psi))
    return out.reshape(x.shape[:-2] + (ell - 1, P.N))


def modup_level(x: np.ndarray, P: Params) -> np.ndarray:
    """[ell][N] coefficient form -> [ceil(ell/alpha)][ell+K][N] on the basis q_0..q_{ell-1}, p_0..p_{K-1}."""
    x = np.ascontiguousarray(x, dtype=np.uint64)
    ell = x.shape[0]
    vp = _arr_u64(P.primes[:ell] + P.primes[P.L:])
    beta = -(-ell // P.alpha)
    out = np.empty((beta, ell + P.K, P.N), dtype=np.uint64)
    lib().orc_modup_level(_ptr(x), _ptr(out), _u32(P.logN), _u32(ell), _u32(P.K), _u32(P.alpha), _ptr(vp))
    return out


def keyswitch_level(d: np.ndarray, key: np.ndarray, P: Params) -> np.ndarray:
    """d [ell][N] eval, full-level key [dnum][2][L+K][N] -> [2][ell][N] eval."""
    d = np.ascontiguousarray(d, dtype=np.uint64)
    key = np.ascontiguousarray(key, dtype=np.uint64)
    ell = d.shape[0]
    assert d.shape == (ell, P.N) and key.shape == (P.dnum, 2, P.L + P.K, P.N)
    out = np.empty((2, ell, P.N), dtype=np.uint64)
    lib().orc_keyswitch_level(_ptr(d), _ptr(key), _ptr(out), *_level_tail(P, ell))
    return out


def hmult_relin_level(ct1: np.ndarray, ct2: np.ndarray, evk: np.ndarray, P: Params) -> np.ndarray:
    ct1 = np.ascontiguousarray(ct1, dtype=np.uint64)
    ct2 = np.ascontiguousarray(ct2, dtype=np.uint64)
    evk = np.ascontiguousarray(evk, dtype=np.uint64)
    ell = ct1.shape[1]
    assert ct1.shape == ct2.shape == (2, ell, P.N) and evk.shape == (P.dnum, 2, P.L + P.K, P.N)
    out = np.empty((2, ell, P.N), dtype=np.uint64)
    lib().orc_hmult_relin_level(_ptr(ct1), _ptr(ct2), _ptr(evk), _ptr(out), *_level_tail(P, ell))
    return out


def hrot_level(ct: np.ndarray, g: int, rk: np.ndarray, P: Params) -> np.ndarray:
    ct = np.ascontiguousarray(ct, dtype=np.uint64)
    rk = np.ascontiguousarray(rk, dtype=np.uint64)
    ell = ct.shape[1]
    assert ct.shape == (2, ell, P.N) and rk.shape == (P.dnum, 2, P.L + P.K, P.N)
    out = np.empty((2, ell, P.N), dtype=np.uint64)
    lib().orc_hrot_level(_ptr(ct), _u32(g), _ptr(rk), _ptr(out), *_level_tail(P, ell))
    return out


def hrot_hoisted_mac_level(ct: np.ndarray, galois: Sequence[int], rks: Sequence[np.ndarray], pt: np.ndarray,
                           P: Params) -> np.ndarray:
    """ct [2][ell][N]; full-level keys; pt [n_rot][ell][N] -> [2][ell][N]."""
    ct = np.ascontiguousarray(ct, dtype=np.uint64)
    pt = np.ascontiguousarray(pt, dtype=np.uint64)
    n_rot, ell = len(galois), ct.shape[1]
    assert len(rks) == n_rot and pt.shape == (n_rot, ell, P.N) and ct.shape == (2, ell, P.N)
    rks = [np.ascontiguousarray(k, dtype=np.uint64) for k in rks]
    ptrs = (ctypes.c_void_p * n_rot)(*[k.ctypes.data for k in rks])
    g = np.ascontiguousarray(np.array(galois, dtype=np.uint32))
    out = np.empty((2, ell, P.N), dtype=np.uint64)
    lib().orc_hrot_hoisted_mac_level(_ptr(ct), _u32(n_rot), _ptr(g), ptrs, _ptr(pt), _ptr(out), *_level_tail(P, ell))
    return out


def hrot_dh_mac_level(ct: np.ndarray, galois: Sequence[int], rks: Sequence[np.ndarray], pt: np.ndarray,
                      P: Params) -> np.ndarray:
    """Double-hoisted rotate-MAC.  ct [2][ell][N]; full-level keys; pt [n_rot][ell+K][N] (the level's
    extended basis: q_0..q_{ell-1}, p_0..p_{K-1}) -> [2][ell][N]."""
    ct = np.ascontiguousarray(ct, dtype=np.uint64)
    pt = np.ascontiguousarray(pt, dtype=np.uint64)
    n_rot, ell = len(galois), ct.shape[1]
    assert len(rks) == n_rot and pt.shape == (n_rot, ell + P.K, P.N) and ct.shape == (2, ell, P.N)
    rks = [np.ascontiguousarray(k, dtype=np.uint64) for k in rks]
    ptrs = (ctypes.c_void_p * n_rot)(*[k.ctypes.data for k in rks])
    g = np.ascontiguousarray(np.array(galois, dtype=np.uint32))
    out = np.empty((2, ell, P.N), dtype=np.uint64)
    lib().orc_hrot_dh_mac_level(_ptr(ct), _u32(n_rot), _ptr(g), ptrs, _ptr(pt), _ptr(out), *_level_tail(P, ell))
    return out


def dh_mac_noise_bound(P: Params, s_l1: int, pt_l1_sum: int, level: Optional[int] = None) -> int:
    """ceil(sum_r ||pt_r||_1 * beta * N * alpha * max_j Q_j * 19 / P) + K * (1 + ||s||_1) + 1."""
    ell = P.L if level is None else level
    qs, ps = P.primes[:ell], P.primes[P.L:]
    Pprod = 1
    for p in ps:
        Pprod *= p
    beta = -(-ell // P.alpha)
    maxQ = 0
    for j in range(beta):
        Qj = 1
        for q in qs[j * P.alpha:(j + 1) * P.alpha]:
            Qj *= q
        maxQ = max(maxQ, Qj)
    first = -((-(pt_l1_sum * beta * P.N * P.alpha * maxQ * 19)) // Pprod)
    return first + P.K * (1 + s_l1) + 1


def moddown_merged(x: np.ndarray, P: Params) -> np.ndarray:
    """[ell+K][N] coefficient form on the level's extended basis -> [ell-1][N]: division by P*q_{ell-1}."""
    x = np.ascontiguousarray(x, dtype=np.uint64)
    ell = x.shape[0] - P.K
    assert 2 <= ell <= P.L
    vp = _arr_u64(P.primes[:ell] + P.primes[P.L:])
    out = np.empty((ell - 1, P.N), dtype=np.uint64)
    lib().orc_moddown_merged(_ptr(x), _ptr(out), _u32(P.logN), _u32(ell), _u32(P.K), _ptr(vp))
    return out


def hmult_relin_rescale_level(ct1: np.ndarray, ct2: np.ndarray, evk: np.ndarray, P: Params) -> np.ndarray:
    """[2][ell][N] x [2][ell][N] -> [2][ell-1][N]: HMult + relinearisation + rescale with one merged division."""
    ct1 = np.ascontiguousarray(ct1, dtype=np.uint64)
    ct2 = np.ascontiguousarray(ct2, dtype=np.uint64)
    evk = np.ascontiguousarray(evk, dtype=np.uint64)
    ell = ct1.shape[1]
    assert ell >= 2 and ct1.shape == ct2.shape == (2, ell, P.N) and evk.shape == (P.dnum, 2, P.L + P.K, P.N)
    out = np.empty((2, ell - 1, P.N), dtype=np.uint64)
    lib().orc_hmult_relin_rescale_level(_ptr(ct1), _ptr(ct2), _ptr(evk), _ptr(out), *_level_tail(P, ell))
    return out


def hrot_dh_mac_rescale_level(ct: np.ndarray, galois: Sequence[int], rks: Sequence[np.ndarray], pt: np.ndarray,
                              P: Params) -> np.ndarray:
    """Double-hoisted rotate-MAC with the merged ModDown + rescale: [2][ell][N] -> [2][ell-1][N]."""
    ct = np.ascontiguousarray(ct, dtype=np.uint64)
    pt = np.ascontiguousarray(pt, dtype=np.uint64)
    n_rot, ell = len(galois), ct.shape[1]
    assert ell >= 2 and len(rks) == n_rot and pt.shape == (n_rot, ell + P.K, P.N) and ct.shape == (2, ell, P.N)
    rks = [np.ascontiguousarray(k, dtype=np.uint64) for k in rks]
    ptrs = (ctypes.c_void_p * n_rot)(*[k.ctypes.data for k in rks])
    g = np.ascontiguousarray(np.array(galois, dtype=np.uint32))
    out = np.empty((2, ell - 1, P.N), dtype=np.uint64)
    lib().orc_hrot_dh_mac_rescale_level(_ptr(ct), _u32(n_rot), _ptr(g), ptrs, _ptr(pt), _ptr(out),
                                        *_level_tail(P, ell))
    return out


def lintrans_bsgs_level(ct: np.ndarray, baby_galois: Sequence[int], baby_rks: Sequence[np.ndarray],
                        giant_galois: Sequence[int], giant_rks: Sequence[np.ndarray], pt: np.ndarray,
                        P: Params) -> np.ndarray:
    """Baby-step giant-step linear transform as the composition of two defined operations:
         inner_g = double-hoisted rotate-MAC of ct over the baby rotations with plaintexts pt[g][:]
         out     = sum_g HRot(inner_g, giant rotation g)            (limb-wise sum)
    ct [2][ell][N]; pt [n2][n1][ell+K][N]; every rotation, identities included, is a key switch."""
    ct = np.ascontiguousarray(ct, dtype=np.uint64)
    ell = ct.shape[1]
    n1, n2 = len(baby_galois), len(giant_galois)
    assert pt.shape == (n2, n1, ell + P.K, P.N) and len(baby_rks) == n1 and len(giant_rks) == n2
    q = P.primes[:ell]
    out = np.zeros((2, ell, P.N), dtype=np.uint64)
    for g in range(n2):
        inner = hrot_dh_mac_level(ct, baby_galois, baby_rks, np.ascontiguousarray(pt[g]), P)
        rot = hrot_level(inner, giant_galois[g], giant_rks[g], P)
        for t in range(2):
            out[t] = pointwise("add", out[t], rot[t], q)
    return out


# ------------------------------------------------------------- harness helpers
def lift_signed(v: np.ndarray, primes: Sequence[int]) -> np.ndarray:
    """Small signed coefficients [N] -> canonical residues [len(primes)][N]."""
    v = np.asarray(v, dtype=np.int64)
    out = np.empty((len(primes), v.shape[0]), dtype=np.uint64)
    for i, p in enumerate(primes):
        out[i] = np.where(v >= 0, v, v + int(p)).astype(np.uint64)
    return out


def secret_eval(s: np.ndarray, P: Params) -> np.ndarray:
    """Ternary secret [N] (int8) -> evaluation form over all L+K limbs."""
    return ntt_batch(lift_signed(s, P.primes), P, 0)


def pointwise(op: str, a: np.ndarray, b: np.ndarray, primes: Sequence[int]) -> np.ndarray:
    """Limb-wise a (op) b for [n_limbs][N] arrays, op in mul/add/sub."""
    a = np.ascontiguousarray(a, dtype=np.uint64)
    b = np.ascontiguousarray(b, dtype=np.uint64)
    out = np.empty_like(a)
    f = getattr(lib(), "orc_pointwise_" + op)
    n = a.shape[-1]
    for i, p in enumerate(primes):
        f(_ptr(a[i]), _ptr(b[i]), _ptr(out[i]), ctypes.c_size_t(n), _u64(p))
    return out


def make_switch_key(s_hat: np.ndarray, sp_hat: np.ndarray, a: np.ndarray, e: np.ndarray, P: Params) -> np.ndarray:
    """Switching key s' -> s.  a: uniform [dnum][L+K][N]; e: int64 [dnum][N]; returns [dnum][2][L+K][N]."""
    s_hat = np.ascontiguousarray(s_hat, dtype=np.uint64)
    sp_hat = np.ascontiguousarray(sp_hat, dtype=np.uint64)
    a = np.ascontiguousarray(a, dtype=np.uint64)
    e = np.ascontiguousarray(e, dtype=np.int64)
    D = P.L + P.K
    assert s_hat.shape == sp_hat.shape == (D, P.N) and a.shape == (P.dnum, D, P.N) and e.shape == (P.dnum, P.N)
    key = np.empty((P.dnum, 2, D, P.N), dtype=np.uint64)
    lib().orc_make_switch_key(_ptr(s_hat), _ptr(sp_hat), _ptr(a), _ptr(e), _ptr(key), *P._tail())
    return key


def centred_small(x_eval: np.ndarray, P: Params, n_limbs: int) -> np.ndarray:
    """INTT the first n_limbs limbs of an evaluation-form value that is supposed to be SMALL, centre
    every limb to (-q/2, q/2] and require all limbs to agree (then, by CRT, that common value is the
    centred representative modulo the whole product).  Returns the int64 coefficient vector."""
    c = ntt_batch(np.ascontiguousarray(x_eval[:n_limbs]), P, 0, inverse=True)
    ref = None
    for i in range(n_limbs):
        q = P.primes[i]
        v = c[i].astype(np.int64)
        v = np.where(c[i] > np.uint64(q // 2), v - q, v)
        if ref is None:
            ref = v
        elif not np.array_equal(ref, v):
            raise AssertionError(f"limb {i} disagrees with limb 0: value is not small modulo the product")
    return ref


def crt_centred(x_eval: np.ndarray, P: Params, n_limbs: int) -> list:
    """INTT the first n_limbs limbs and reconstruct every coefficient modulo their product with big integers,
    centred to (-Q/2, Q/2]: for values that are small against the product but not against a single limb."""
    c = ntt_batch(np.ascontiguousarray(x_eval[:n_limbs]), P, 0, inverse=True)
    primes = [int(p) for p in P.primes[:n_limbs]]
    Q = 1
    for p in primes:
        Q *= p
    lift = [(Q // p) * pow(Q // p, -1, p) for p in primes]
    out = []
    for k in range(c.shape[1]):
        v = sum(int(c[i, k]) * lift[i] for i in range(n_limbs)) % Q
        out.append(v - Q if v > Q // 2 else v)
    return out


def keyswitch_noise(d: np.ndarray, ks: np.ndarray, s_hat: np.ndarray, sp_hat: np.ndarray, P: Params,
                    level: Optional[int] = None) -> np.ndarray:
    """E = ks0 + ks1*s - d*s'  over the (active) q-limbs, as centred integer coefficients (must be small)."""
    ell = P.L if level is None else level
    q = P.primes[:ell]
    t = pointwise("add", ks[0], pointwise("mul", ks[1], s_hat[:ell], q), q)
    t = pointwise("sub", t, pointwise("mul", d, sp_hat[:ell], q), q)
    return centred_small(t, P, ell)


def keyswitch_noise_bound(P: Params, s_l1: int, level: Optional[int] = None) -> int:
    """ceil(beta * N * alpha * max_j Q_j * 19 / P) + K * (1 + ||s||_1) + 1 over the beta digits of the level."""
    ell = P.L if level is None else level
    qs, ps = P.primes[:ell], P.primes[P.L:]
    Pprod = 1
    for p in ps:
        Pprod *= p
    beta = -(-ell // P.alpha)
    maxQ = 0
    for j in range(beta):
        Qj = 1
        for q in qs[j * P.alpha:(j + 1) * P.alpha]:
            Qj *= q
        maxQ = max(maxQ, Qj)
    first = -((-(beta * P.N * P.alpha * maxQ * 19)) // Pprod)
    return first + P.K * (1 + s_l1) + 1


# ------------------------------------------------- canonical embedding (encoding of slot vectors)
# The CKKS plaintext space (the scheme of the paper's Section 2): a real polynomial m of degree < N is
# identified with its values at zeta_j = exp(i*pi*5^j / N), j < N/2 (one of each conjugate pair of roots
# of X^N + 1) -- the "slots".  X -> X^(5^r) permutes these roots, zeta_j -> zeta_(j+r), so the automorphism
# with Galois element 5^r rotates the slot vector by r places.  Plain O(N^2) definitions in complex128;
# nothing here is shared with the HIP library, which never encodes.
def slot_roots(logN: int) -> np.ndarray:
    """zeta_j = exp(i*pi*(5^j mod 2N)/N) for j < N/2."""
    n = 1 << logN
    e = np.array([pow(5, j, 2 * n) for j in range(n // 2)], dtype=np.float64)
    return np.exp(1j * np.pi * e / n)


def encode(z: np.ndarray, scale: float, logN: int) -> np.ndarray:
    """Slot vector z [N/2] complex -> integer coefficients [N] (int64) of the real polynomial with
    m(zeta_j) = scale * z_j, rounded to nearest: m_k = round(scale * (2/N) * Re(sum_j z_j * conj(zeta_j)^k))."""
    n = 1 << logN
    z = np.asarray(z, dtype=np.complex128)
    assert z.shape == (n // 2,)
    zeta = slot_roots(logN)
    k = np.arange(n, dtype=np.float64)
    # conj(zeta_j)^k, as exp(-i * k * angle_j) to avoid the error growth of repeated products
    ang = np.angle(zeta)
    w = np.exp(-1j * np.outer(k, ang))            # [N][N/2]
    m = (2.0 / n) * np.real(w @ z) * scale
    return np.rint(m).astype(np.int64)


def decode(coeffs: np.ndarray, scale: float, logN: int) -> np.ndarray:
    """Integer coefficients [N] -> slot vector [N/2]: z_j = m(zeta_j) / scale."""
    n = 1 << logN
    c = np.asarray(coeffs, dtype=np.float64)
    ang = np.angle(slot_roots(logN))
    w = np.exp(1j * np.outer(ang, np.arange(n, dtype=np.float64)))   # zeta_j^k, [N/2][N]
    return (w @ c) / scale


def encode_limbs(z: np.ndarray, scale: float, P: Params, limb_primes: Sequence[int], limb_psi: Sequence[int]) -> np.ndarray:
    """encode(), lifted to the given RNS limbs and transformed to evaluation form: [len(limb_primes)][N]."""
    lifted = lift_signed(encode(z, scale, P.logN), limb_primes)
    return np.stack([ntt(lifted[i], P.logN, int(m), int(w)) for i, (m, w) in enumerate(zip(limb_primes, limb_psi))])


def matrix_diagonal(M: np.ndarray, d: int) -> np.ndarray:
    """Generalised diagonal d of an n x n matrix: diag_d[j] = M[j][(j + d) mod n], so that
    M z = sum_d diag_d * rot_d(z) with rot_d(z)[j] = z[(j + d) mod n]."""
    n = M.shape[0]
    j = np.arange(n)
    return M[j, (j + d) % n]


def bsgs_diagonal_plaintexts(M: np.ndarray, n1: int, n2: int, scale: float, P: Params, level: int) -> np.ndarray:
    """Plaintexts [n2][n1][level+K][N] that make lintrans_bsgs_level (baby rotations 0..n1-1, giant rotations
    0, n1, .., (n2-1)*n1) evaluate z -> M z on the slots, for a matrix whose non-zero diagonals are 0 .. n1*n2-1:
      M z = sum_g rot_{g*n1}( sum_b rot_{-g*n1}(diag_{g*n1+b}) * rot_b(z) ),
    so plaintext (g, b) encodes diagonal g*n1 + b rotated by -g*n1."""
    basis = list(P.primes[:level]) + list(P.primes[P.L:])
    psis = list(P.psi[:level]) + list(P.psi[P.L:])
    out = np.empty((n2, n1, len(basis), P.N), dtype=np.uint64)
    for g in range(n2):
        for b in range(n1):
            diag = np.roll(matrix_diagonal(M, g * n1 + b), g * n1)   # rot_{-g*n1}: entry j takes entry j - g*n1
            out[g, b] = encode_limbs(diag, scale, P, basis, psis)
    return out
