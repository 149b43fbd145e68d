"""Thin ctypes binding of libckks_mi355x.so (the C ABI in include/ckks_mi355x.h).

Argument marshalling only: every step of the key-switch path runs in the HIP
kernels of the library.  PyTorch supplies device memory (tensors of dtype
uint64 / int64, passed as raw pointers) and the current HIP stream.  There is no
CPU fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch  # imported first so that the library binds to the HIP runtime torch already loaded

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libckks_mi355x.so")

CKKS_OK, CKKS_EINVAL, CKKS_EUNSUPPORTED, CKKS_EHIP, CKKS_ENOMEM = 0, -1, -2, -3, -4
ROTATIONS_PER_LAUNCH = 16
(OP_NTT, OP_MODUP, OP_MODDOWN, OP_AUTOMORPH, OP_KEYSWITCH, OP_HMULT_RELIN, OP_HROT, OP_HROT_HOISTED_MAC,
 OP_RESCALE, OP_HROT_DH_MAC) = range(10)
PW_ADD, PW_SUB, PW_MUL, PW_MAC = range(4)  # CKKS_PW_* of ckks_pointwise

EXPORTS = (
    "ckks_table_bytes", "ckks_ctx_create", "ckks_ctx_destroy", "ckks_last_error", "ckks_ctx_psi",
    "ckks_workspace_bytes", "ckks_ntt", "ckks_intt", "ckks_modup", "ckks_moddown", "ckks_automorph",
    "ckks_keyswitch", "ckks_hmult_relin", "ckks_hrot", "ckks_hrot_hoisted_mac",
    "ckks_profile_enable", "ckks_profile_read", "ckks_set_overlap",
    "ckks_workspace_bytes_at", "ckks_keyswitch_at", "ckks_hmult_relin_at", "ckks_hrot_at",
    "ckks_hrot_hoisted_mac_at", "ckks_rescale", "ckks_hrot_dh_mac", "ckks_hrot_dh_mac_at",
    "ckks_hmult_relin_rescale_at", "ckks_hrot_dh_mac_rescale_at",
    "ckks_lintrans_bsgs_workspace_bytes", "ckks_lintrans_bsgs_at", "ckks_hrot_multi_at", "ckks_pointwise",
    "ckks_rescale_static",
)
STATIC_SCRATCH_BYTES = 32 << 20

_u32, _u64, _int, _sz, _vp = ctypes.c_uint32, ctypes.c_uint64, ctypes.c_int, ctypes.c_size_t, ctypes.c_void_p
_lib = None


class CkksError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"ckks error {code}: {msg}")
        self.code = code


def load() -> ctypes.CDLL:
    """Load the built library (never builds, never falls back)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: run `python __graft_entry__.py build` "
                           "(or paper_2310_16530_amd/build.py) first; there is no CPU fallback")
    lib = ctypes.CDLL(LIB_PATH)
    lib.ckks_table_bytes.argtypes = [_u32, _u32, _u32, _u32, ctypes.POINTER(_sz)]
    lib.ckks_ctx_create.argtypes = [ctypes.POINTER(_vp), _u32, _u32, _u32, _u32, _vp, _vp, _vp, _sz, _vp]
    lib.ckks_ctx_destroy.argtypes = [_vp]
    lib.ckks_ctx_destroy.restype = None
    lib.ckks_last_error.argtypes = [_vp]
    lib.ckks_last_error.restype = ctypes.c_char_p
    lib.ckks_ctx_psi.argtypes = [_vp, _u32]
    lib.ckks_ctx_psi.restype = _u64
    lib.ckks_workspace_bytes.argtypes = [_vp, _int, _u32, ctypes.POINTER(_sz)]
    lib.ckks_ntt.argtypes = [_vp, _vp, _u32, _u32, _u32, _vp]
    lib.ckks_intt.argtypes = [_vp, _vp, _u32, _u32, _u32, _vp]
    lib.ckks_modup.argtypes = [_vp, _vp, _vp, _u32, _vp]
    lib.ckks_moddown.argtypes = [_vp, _vp, _vp, _u32, _vp]
    lib.ckks_automorph.argtypes = [_vp, _vp, _vp, _u32, _u32, _u32, _int, _u32, _vp]
    lib.ckks_keyswitch.argtypes = [_vp, _vp, _vp, _vp, _u32, _vp, _sz, _vp]
    lib.ckks_hmult_relin.argtypes = [_vp, _vp, _vp, _vp, _vp, _u32, _vp, _sz, _vp]
    lib.ckks_hrot.argtypes = [_vp, _vp, _u32, _vp, _vp, _u32, _vp, _sz, _vp]
    lib.ckks_hrot_hoisted_mac.argtypes = [_vp, _vp, _u32, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
    lib.ckks_set_overlap.argtypes = [_vp, _int]
    lib.ckks_workspace_bytes_at.argtypes = [_vp, _int, _u32, _u32, ctypes.POINTER(_sz)]
    lib.ckks_keyswitch_at.argtypes = [_vp, _u32, _vp, _vp, _vp, _u32, _vp, _sz, _vp]
    lib.ckks_hmult_relin_at.argtypes = [_vp, _u32, _vp, _vp, _vp, _vp, _u32, _vp, _sz, _vp]
    lib.ckks_hrot_at.argtypes = [_vp, _u32, _vp, _u32, _vp, _vp, _u32, _vp, _sz, _vp]
    lib.ckks_hrot_hoisted_mac_at.argtypes = [_vp, _u32, _vp, _u32, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
    lib.ckks_rescale.argtypes = [_vp, _u32, _vp, _vp, _u32, _vp, _sz, _vp]
    lib.ckks_rescale_static.argtypes = [_vp, _u32, _vp, _vp, _u32, _vp]
    lib.ckks_hrot_dh_mac.argtypes = [_vp, _vp, _u32, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
    lib.ckks_hrot_dh_mac_at.argtypes = [_vp, _u32, _vp, _u32, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
    lib.ckks_hmult_relin_rescale_at.argtypes = [_vp, _u32, _vp, _vp, _vp, _vp, _u32, _vp, _sz, _vp]
    lib.ckks_hrot_dh_mac_rescale_at.argtypes = [_vp, _u32, _vp, _u32, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
    lib.ckks_hrot_multi_at.argtypes = [_vp, _u32, _vp, _vp, _vp, _vp, _u32, _vp, _sz, _vp]
    lib.ckks_pointwise.argtypes = [_vp, _int, _vp, _vp, _vp, _u32, _u32, _u32, _u32, _vp]
    lib.ckks_lintrans_bsgs_workspace_bytes.argtypes = [_vp, _u32, _u32, _u32, ctypes.POINTER(_sz)]
    lib.ckks_lintrans_bsgs_at.argtypes = [_vp, _u32, _vp, _u32, _vp, _vp, _u32, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
    lib.ckks_profile_enable.argtypes = [_vp, _int]
    lib.ckks_profile_read.argtypes = [_vp, _u32, ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(_u64),
                                      ctypes.POINTER(ctypes.c_double), ctypes.POINTER(_u64)]
    for name in EXPORTS:
        f = getattr(lib, name)
        if name not in ("ckks_ctx_destroy", "ckks_last_error", "ckks_ctx_psi"):
            f.restype = _int
    _lib = lib
    return lib


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev_ptr(t: torch.Tensor) -> int:
    if not t.is_cuda or not t.is_contiguous() or t.element_size() != 8:
        raise ValueError("expected a contiguous 64-bit device tensor")
    return t.data_ptr()


def check_operand(t: torch.Tensor, words: int, what: str, device: Optional[torch.device] = None) -> int:
    """The C ABI takes raw pointers and cannot see buffer lengths, so every operand is checked here before any
    launch: 64-bit elements, contiguous, exactly `words` of them, on `device`.  Returns the device pointer."""
    if not isinstance(t, torch.Tensor) or t.element_size() != 8 or t.is_floating_point():
        raise ValueError(f"{what}: expected a tensor of 64-bit integers")
    if not t.is_contiguous():
        raise ValueError(f"{what}: tensor is not contiguous")
    if t.numel() != words:
        raise ValueError(f"{what}: expected {words} words, got {t.numel()} (shape {tuple(t.shape)})")
    if not t.is_cuda or (device is not None and t.device != device):
        raise ValueError(f"{what}: tensor is on {t.device}, the context is on {device}")
    return t.data_ptr()


def check_batch(t: torch.Tensor, words_per_item: int, what: str) -> int:
    """Number of items in t when each takes words_per_item words; rejects sizes that are no whole multiple."""
    n = t.numel()
    if words_per_item <= 0 or n == 0 or n % words_per_item:
        raise ValueError(f"{what}: {n} words is not a positive multiple of {words_per_item}")
    return n // words_per_item


def check_chain(L: int, K: int, primes: Sequence[int], psi: Optional[Sequence[int]]) -> None:
    """The library reads L + K primes (and roots) from the host arrays it is handed."""
    if len(primes) != L + K:
        raise ValueError(f"expected L + K = {L + K} primes, got {len(primes)}")
    if psi is not None and len(psi) != L + K:
        raise ValueError(f"expected L + K = {L + K} roots, got {len(psi)}")


class Context:
    """Owns the opaque ckks_ctx, its device tables and one workspace tensor per torch stream (all allocated
    through torch).  Calls made under different current streams get different workspaces, so they may overlap;
    calls on one stream share a workspace and are ordered by the stream.  Every tensor argument is checked for
    dtype, contiguity, exact size and device before the library is called (ValueError, nothing launched)."""

    def __init__(self, logN: int, L: int, K: int, dnum: int, primes: Sequence[int],
                 psi: Optional[Sequence[int]] = None, device: str = "cuda:0"):
        check_chain(L, K, primes, psi)
        lib = load()
        self.logN, self.L, self.K, self.dnum = logN, L, K, dnum
        self.N, self.D = 1 << logN, L + K
        self.device = torch.device(device)
        if self.device.index is None:
            self.device = torch.device(self.device.type, torch.cuda.current_device())
        nbytes = _sz()
        rc = lib.ckks_table_bytes(logN, L, K, dnum, ctypes.byref(nbytes))
        if rc:
            raise CkksError(rc, "ckks_table_bytes rejected the shape")
        self.tables = torch.empty(nbytes.value, dtype=torch.uint8, device=self.device)
        pr = (ctypes.c_uint64 * len(primes))(*[int(p) for p in primes])
        ps = (ctypes.c_uint64 * len(psi))(*[int(p) for p in psi]) if psi is not None else None
        handle = _vp()
        with torch.cuda.device(self.device):
            rc = lib.ckks_ctx_create(ctypes.byref(handle), logN, L, K, dnum, ctypes.cast(pr, _vp),
                                     ctypes.cast(ps, _vp) if ps is not None else None,
                                     self.tables.data_ptr(), nbytes.value, _stream())
        if rc:
            raise CkksError(rc, "ckks_ctx_create failed")
        self.handle = handle
        self._ws = {}

    def __del__(self):
        h = getattr(self, "handle", None)
        if h:
            self.handle = None
            try:
                load().ckks_ctx_destroy(h)
            except Exception:  # interpreter shutdown: module globals may already be gone
                pass

    # -- helpers ---------------------------------------------------------------------
    def _check(self, rc: int):
        if rc:
            raise CkksError(rc, load().ckks_last_error(self.handle).decode())

    def psi(self, i: int) -> int:
        return int(load().ckks_ctx_psi(self.handle, i))

    def workspace_bytes(self, op: int, batch_or_nrot: int) -> int:
        n = _sz()
        self._check(load().ckks_workspace_bytes(self.handle, op, batch_or_nrot, ctypes.byref(n)))
        return n.value

    def workspace_bytes_at(self, op: int, level: int, batch_or_nrot: int) -> int:
        n = _sz()
        self._check(load().ckks_workspace_bytes_at(self.handle, op, level, batch_or_nrot, ctypes.byref(n)))
        return n.value

    def _ws_for(self, need: int) -> torch.Tensor:
        """Workspace of the current torch stream.  A tensor that is replaced by a larger one goes back to torch's
        caching allocator, which hands it out again only in stream order of the stream it was allocated on -- the
        same stream every earlier use of it was enqueued on."""
        key = _stream()
        ws = self._ws.get(key)
        if ws is None or ws.numel() < need:
            self._ws.pop(key, None)
            ws = torch.empty(max(need, 256), dtype=torch.uint8, device=self.device)
            self._ws[key] = ws
        return ws

    def workspace(self, op: int, batch_or_nrot: int, level: Optional[int] = None) -> torch.Tensor:
        need = (self.workspace_bytes(op, batch_or_nrot) if level is None
                else self.workspace_bytes_at(op, level, batch_or_nrot))
        return self._ws_for(need)

    # -- operand checks --------------------------------------------------------------
    def _level(self, level: Optional[int]) -> int:
        ell = self.L if level is None else int(level)
        if not 1 <= ell <= self.L:
            raise ValueError(f"level must be between 1 and L = {self.L}")
        return ell

    def _op(self, t: torch.Tensor, words: int, what: str) -> int:
        return check_operand(t, words, what, self.device)

    def _key(self, k: torch.Tensor, what: str = "key") -> int:
        """Switching keys are always laid out over the whole chain: [dnum][2][L+K][N], also below level L."""
        return self._op(k, self.dnum * 2 * self.D * self.N, what)

    def _keys(self, ks: Sequence[torch.Tensor], n: int, galois: Sequence[int]):
        if len(ks) != n or len(galois) != n or n == 0:
            raise ValueError("one Galois element and one key per rotation, at least one rotation")
        g = (ctypes.c_uint32 * n)(*[int(x) for x in galois])
        ptrs = (ctypes.c_void_p * n)(*[self._key(k, f"key {i}") for i, k in enumerate(ks)])
        return g, ptrs

    def _out(self, out: Optional[torch.Tensor], shape, like: torch.Tensor) -> torch.Tensor:
        return torch.empty(tuple(shape), dtype=like.dtype, device=like.device) if out is None else out

    def set_overlap(self, on: bool) -> None:
        self._check(load().ckks_set_overlap(self.handle, 1 if on else 0))

    def profile_enable(self, on: bool) -> None:
        self._check(load().ckks_profile_enable(self.handle, 1 if on else 0))

    def profile_read(self) -> dict:
        """{kernel name: (launches, total_ms, algorithmic_bytes)} since profile_enable(True)."""
        out = {}
        index = 0
        while True:
            name, n, ms, nbytes = ctypes.c_char_p(), _u64(), ctypes.c_double(), _u64()
            rc = load().ckks_profile_read(self.handle, index, ctypes.byref(name), ctypes.byref(n),
                                          ctypes.byref(ms), ctypes.byref(nbytes))
            if rc:
                break
            out[name.value.decode()] = (n.value, ms.value, nbytes.value)
            index += 1
        return out

    # -- entry points (same names as the C ABI, minus the prefix) ----------------------
    def ntt(self, x: torch.Tensor, prime_first: int = 0, inverse: bool = False) -> torch.Tensor:
        """In place on x = [batch...][n_limbs][N]."""
        if x.dim() < 2 or x.shape[-1] != self.N:
            raise ValueError("x: expected [...][n_limbs][N]")
        n_limbs = x.shape[-2]
        if prime_first < 0 or prime_first + n_limbs > self.D:
            raise ValueError("limb range exceeds the prime chain")
        batch = check_batch(x, n_limbs * self.N, "x")
        f = load().ckks_intt if inverse else load().ckks_ntt
        self._check(f(self.handle, self._op(x, batch * n_limbs * self.N, "x"), prime_first, n_limbs, batch, _stream()))
        return x

    def intt(self, x: torch.Tensor, prime_first: int = 0) -> torch.Tensor:
        return self.ntt(x, prime_first, inverse=True)

    def modup(self, x: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        batch = check_batch(x, self.L * self.N, "x")
        out = self._out(out, tuple(x.shape[:-2]) + (self.dnum, self.D, self.N), x)
        self._check(load().ckks_modup(self.handle, self._op(x, batch * self.L * self.N, "x"),
                                      self._op(out, batch * self.dnum * self.D * self.N, "out"), batch, _stream()))
        return out

    def moddown(self, x: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        batch = check_batch(x, self.D * self.N, "x")
        out = self._out(out, tuple(x.shape[:-2]) + (self.L, self.N), x)
        self._check(load().ckks_moddown(self.handle, self._op(x, batch * self.D * self.N, "x"),
                                        self._op(out, batch * self.L * self.N, "out"), batch, _stream()))
        return out

    def automorph(self, x: torch.Tensor, galois: int, eval_domain: bool, prime_first: int = 0,
                  out: Optional[torch.Tensor] = None) -> torch.Tensor:
        if x.dim() < 2 or x.shape[-1] != self.N:
            raise ValueError("x: expected [...][n_limbs][N]")
        n_limbs = x.shape[-2]
        batch = check_batch(x, n_limbs * self.N, "x")
        out = self._out(out, x.shape, x)
        self._check(load().ckks_automorph(self.handle, self._op(x, x.numel(), "x"), self._op(out, x.numel(), "out"),
                                          prime_first, n_limbs, galois, 1 if eval_domain else 0, batch, _stream()))
        return out

    def pointwise(self, op: int, a: torch.Tensor, b: torch.Tensor, out: Optional[torch.Tensor] = None,
                  prime_first: int = 0) -> torch.Tensor:
        """a (op) b limb by limb; a [..][n_limbs][N], b the same or fewer leading groups (applied cyclically).
        PW_MAC accumulates into `out`, which may be `a` or `b` for the other operations."""
        if a.dim() < 2 or b.dim() < 2 or a.shape[-1] != self.N or b.shape[-1] != self.N:
            raise ValueError("operands: expected [...][n_limbs][N]")
        n_limbs = a.shape[-2]
        batch = check_batch(a, n_limbs * self.N, "a")
        b_period = check_batch(b, n_limbs * self.N, "b")
        if out is None:
            if op == PW_MAC:
                raise ValueError("PW_MAC accumulates into out")
            out = torch.empty_like(a)
        if b.shape[-2] != n_limbs or out.shape != a.shape:
            raise ValueError("operand shapes do not match")
        self._check(load().ckks_pointwise(self.handle, op, self._op(a, a.numel(), "a"), self._op(b, b.numel(), "b"),
                                          self._op(out, a.numel(), "out"), prime_first, n_limbs, batch, b_period,
                                          _stream()))
        return out

    def keyswitch(self, d: torch.Tensor, key: torch.Tensor, out: Optional[torch.Tensor] = None,
                  level: Optional[int] = None) -> torch.Tensor:
        ell = self._level(level)
        batch = check_batch(d, ell * self.N, "d")
        out = self._out(out, tuple(d.shape[:-2]) + (2, ell, self.N), d)
        ws = self.workspace(OP_KEYSWITCH, batch, ell)
        args = (self._op(d, batch * ell * self.N, "d"), self._key(key), self._op(out, batch * 2 * ell * self.N, "out"),
                batch, ws.data_ptr(), ws.numel(), _stream())
        lib = load()
        self._check(lib.ckks_keyswitch(self.handle, *args) if level is None else lib.ckks_keyswitch_at(self.handle, ell, *args))
        return out

    def hmult_relin(self, ct1: torch.Tensor, ct2: torch.Tensor, evk: torch.Tensor,
                    out: Optional[torch.Tensor] = None, level: Optional[int] = None) -> torch.Tensor:
        ell = self._level(level)
        batch = check_batch(ct1, 2 * ell * self.N, "ct1")
        words = batch * 2 * ell * self.N
        out = self._out(out, ct1.shape, ct1)
        ws = self.workspace(OP_HMULT_RELIN, batch, ell)
        args = (self._op(ct1, words, "ct1"), self._op(ct2, words, "ct2"), self._key(evk, "evk"), self._op(out, words, "out"),
                batch, ws.data_ptr(), ws.numel(), _stream())
        lib = load()
        self._check(lib.ckks_hmult_relin(self.handle, *args) if level is None
                    else lib.ckks_hmult_relin_at(self.handle, ell, *args))
        return out

    def hrot(self, ct: torch.Tensor, galois: int, rk: torch.Tensor, out: Optional[torch.Tensor] = None,
             level: Optional[int] = None) -> torch.Tensor:
        ell = self._level(level)
        batch = check_batch(ct, 2 * ell * self.N, "ct")
        words = batch * 2 * ell * self.N
        out = self._out(out, ct.shape, ct)
        ws = self.workspace(OP_HROT, batch, ell)
        args = (self._op(ct, words, "ct"), galois, self._key(rk, "rk"), self._op(out, words, "out"), batch,
                ws.data_ptr(), ws.numel(), _stream())
        lib = load()
        self._check(lib.ckks_hrot(self.handle, *args) if level is None else lib.ckks_hrot_at(self.handle, ell, *args))
        return out

    def hrot_hoisted_mac(self, ct: torch.Tensor, galois: Sequence[int], rks: Sequence[torch.Tensor],
                         pt: torch.Tensor, out: Optional[torch.Tensor] = None,
                         level: Optional[int] = None) -> torch.Tensor:
        """ct [2][level][N], pt [n_rot][level][N]; out = sum_r pt_r * HRot_r(ct) with the decomposition hoisted."""
        ell = self._level(level)
        n_rot = len(galois)
        g, ptrs = self._keys(rks, n_rot, galois)
        words = 2 * ell * self.N
        out = self._out(out, ct.shape, ct)
        ws = self.workspace(OP_HROT_HOISTED_MAC, n_rot, ell)
        args = (self._op(ct, words, "ct"), n_rot, ctypes.cast(g, _vp), ctypes.cast(ptrs, _vp),
                self._op(pt, n_rot * ell * self.N, "pt"), self._op(out, words, "out"), ws.data_ptr(), ws.numel(), _stream())
        lib = load()
        self._check(lib.ckks_hrot_hoisted_mac(self.handle, *args) if level is None
                    else lib.ckks_hrot_hoisted_mac_at(self.handle, ell, *args))
        return out

    # -- levels below L: tensors carry `level` limbs instead of L; keys stay full-level ----------
    def keyswitch_at(self, level: int, d: torch.Tensor, key: torch.Tensor,
                     out: Optional[torch.Tensor] = None) -> torch.Tensor:
        return self.keyswitch(d, key, out, level)

    def hmult_relin_at(self, level: int, ct1: torch.Tensor, ct2: torch.Tensor, evk: torch.Tensor,
                       out: Optional[torch.Tensor] = None) -> torch.Tensor:
        return self.hmult_relin(ct1, ct2, evk, out, level)

    def hrot_at(self, level: int, ct: torch.Tensor, galois: int, rk: torch.Tensor,
                out: Optional[torch.Tensor] = None) -> torch.Tensor:
        return self.hrot(ct, galois, rk, out, level)

    def hrot_hoisted_mac_at(self, level: int, ct: torch.Tensor, galois: Sequence[int], rks: Sequence[torch.Tensor],
                            pt: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        return self.hrot_hoisted_mac(ct, galois, rks, pt, out, level)

    def rescale(self, level: int, ct: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """ct [batch...][2][level][N] -> [batch...][2][level-1][N]."""
        ell = self._level(level)
        if ell < 2:
            raise ValueError("rescale needs at least two limbs")
        batch = check_batch(ct, 2 * ell * self.N, "ct")
        out = self._out(out, tuple(ct.shape[:-2]) + (ell - 1, self.N), ct)
        ws = self.workspace(OP_RESCALE, batch, ell)
        self._check(load().ckks_rescale(self.handle, ell, self._op(ct, batch * 2 * ell * self.N, "ct"),
                                        self._op(out, batch * 2 * (ell - 1) * self.N, "out"), batch,
                                        ws.data_ptr(), ws.numel(), _stream()))
        return out

    def rescale_static(self, level: int, ct: torch.Tensor, out: torch.Tensor) -> torch.Tensor:
        """ckks_rescale with the library's static scratch as workspace; the caller brings `out` (nothing is allocated)."""
        ell = self._level(level)
        if ell < 2:
            raise ValueError("rescale needs at least two limbs")
        batch = check_batch(ct, 2 * ell * self.N, "ct")
        self._check(load().ckks_rescale_static(self.handle, ell, self._op(ct, batch * 2 * ell * self.N, "ct"),
                                               self._op(out, batch * 2 * (ell - 1) * self.N, "out"), batch, _stream()))
        return out

    def hrot_dh_mac(self, ct: torch.Tensor, galois: Sequence[int], rks: Sequence[torch.Tensor], pt: torch.Tensor,
                    out: Optional[torch.Tensor] = None, level: Optional[int] = None) -> torch.Tensor:
        """Double-hoisted rotate-MAC; pt [n_rot][level+K][N] on the level's extended basis."""
        ell = self._level(level)
        n_rot = len(galois)
        g, ptrs = self._keys(rks, n_rot, galois)
        words = 2 * ell * self.N
        out = self._out(out, ct.shape, ct)
        ws = self.workspace(OP_HROT_DH_MAC, n_rot, ell)
        args = (self._op(ct, words, "ct"), n_rot, ctypes.cast(g, _vp), ctypes.cast(ptrs, _vp),
                self._op(pt, n_rot * (ell + self.K) * self.N, "pt"), self._op(out, words, "out"),
                ws.data_ptr(), ws.numel(), _stream())
        if level is None:
            rc = load().ckks_hrot_dh_mac(self.handle, *args)
        else:
            rc = load().ckks_hrot_dh_mac_at(self.handle, ell, *args)
        self._check(rc)
        return out

    # -- ModDown merged with the following rescale: outputs carry level - 1 limbs -----------------
    def hmult_relin_rescale_at(self, level: int, ct1: torch.Tensor, ct2: torch.Tensor, evk: torch.Tensor,
                               out: Optional[torch.Tensor] = None) -> torch.Tensor:
        ell = self._level(level)
        if ell < 2:
            raise ValueError("rescale needs at least two limbs")
        batch = check_batch(ct1, 2 * ell * self.N, "ct1")
        words = batch * 2 * ell * self.N
        out = self._out(out, tuple(ct1.shape[:-2]) + (ell - 1, self.N), ct1)
        ws = self.workspace(OP_HMULT_RELIN, batch, ell)
        self._check(load().ckks_hmult_relin_rescale_at(self.handle, ell, self._op(ct1, words, "ct1"),
                                                       self._op(ct2, words, "ct2"), self._key(evk, "evk"),
                                                       self._op(out, batch * 2 * (ell - 1) * self.N, "out"), batch,
                                                       ws.data_ptr(), ws.numel(), _stream()))
        return out

    def hrot_dh_mac_rescale_at(self, level: int, ct: torch.Tensor, galois: Sequence[int], rks: Sequence[torch.Tensor],
                               pt: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        ell = self._level(level)
        if ell < 2:
            raise ValueError("rescale needs at least two limbs")
        n_rot = len(galois)
        g, ptrs = self._keys(rks, n_rot, galois)
        out = self._out(out, (2, ell - 1, self.N), ct)
        ws = self.workspace(OP_HROT_DH_MAC, n_rot, ell)
        self._check(load().ckks_hrot_dh_mac_rescale_at(self.handle, ell, self._op(ct, 2 * ell * self.N, "ct"), n_rot,
                                                       ctypes.cast(g, _vp), ctypes.cast(ptrs, _vp),
                                                       self._op(pt, n_rot * (ell + self.K) * self.N, "pt"),
                                                       self._op(out, 2 * (ell - 1) * self.N, "out"),
                                                       ws.data_ptr(), ws.numel(), _stream()))
        return out

    def lintrans_bsgs_at(self, level: int, ct: torch.Tensor, baby_galois: Sequence[int], baby_rks: Sequence[torch.Tensor],
                         giant_galois: Sequence[int], giant_rks: Sequence[torch.Tensor], pt: torch.Tensor,
                         out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """pt [n2][n1][level+K][N]; out = sum_g HRot_g(sum_b pt[g][b] * HRot_b(ct)), baby steps double-hoisted."""
        ell = self._level(level)
        n1, n2 = len(baby_galois), len(giant_galois)
        bg, bk = self._keys(baby_rks, n1, baby_galois)
        gg, gk = self._keys(giant_rks, n2, giant_galois)
        words = 2 * ell * self.N
        out = self._out(out, ct.shape, ct)
        need = _sz()
        self._check(load().ckks_lintrans_bsgs_workspace_bytes(self.handle, ell, n1, n2, ctypes.byref(need)))
        ws = self._ws_for(need.value)
        self._check(load().ckks_lintrans_bsgs_at(self.handle, ell, self._op(ct, words, "ct"), n1, ctypes.cast(bg, _vp),
                                                 ctypes.cast(bk, _vp), n2, ctypes.cast(gg, _vp), ctypes.cast(gk, _vp),
                                                 self._op(pt, n1 * n2 * (ell + self.K) * self.N, "pt"),
                                                 self._op(out, words, "out"), ws.data_ptr(), ws.numel(), _stream()))
        return out

    def hrot_multi_at(self, level: int, ct: torch.Tensor, galois: Sequence[int], rks: Sequence[torch.Tensor],
                      out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """ct [batch][2][level][N]; instance b is rotated by galois[b] with key rks[b]."""
        ell = self._level(level)
        batch = len(galois)
        g, ptrs = self._keys(rks, batch, galois)
        words = batch * 2 * ell * self.N
        out = self._out(out, ct.shape, ct)
        ws = self.workspace(OP_HROT, min(batch, ROTATIONS_PER_LAUNCH), ell)
        self._check(load().ckks_hrot_multi_at(self.handle, ell, self._op(ct, words, "ct"), ctypes.cast(g, _vp),
                                              ctypes.cast(ptrs, _vp), self._op(out, words, "out"), batch,
                                              ws.data_ptr(), ws.numel(), _stream()))
        return out
