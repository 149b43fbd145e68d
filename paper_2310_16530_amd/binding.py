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
)

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


class Context:
    """Owns the opaque ckks_ctx, its device tables and a workspace tensor (all allocated through torch)."""

    def __init__(self, logN: int, L: int, K: int, dnum: int, primes: Sequence[int],
                 psi: Optional[Sequence[int]] = None, device: str = "cuda:0"):
        lib = load()
        self.logN, self.L, self.K, self.dnum = logN, L, K, dnum
        self.N, self.D = 1 << logN, L + K
        self.device = torch.device(device)
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
        self._ws = None

    def __del__(self):
        h = getattr(self, "handle", None)
        if h:
            load().ckks_ctx_destroy(h)
            self.handle = None

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

    def workspace(self, op: int, batch_or_nrot: int, level: Optional[int] = None) -> torch.Tensor:
        need = (self.workspace_bytes(op, batch_or_nrot) if level is None
                else self.workspace_bytes_at(op, level, batch_or_nrot))
        if self._ws is None or self._ws.numel() < need:
            self._ws = None
            self._ws = torch.empty(max(need, 256), dtype=torch.uint8, device=self.device)
        return self._ws

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
        n_limbs = x.shape[-2]
        batch = x.numel() // (n_limbs * self.N)
        f = load().ckks_intt if inverse else load().ckks_ntt
        self._check(f(self.handle, _dev_ptr(x), prime_first, n_limbs, batch, _stream()))
        return x

    def intt(self, x: torch.Tensor, prime_first: int = 0) -> torch.Tensor:
        return self.ntt(x, prime_first, inverse=True)

    def modup(self, x: torch.Tensor) -> torch.Tensor:
        batch = x.numel() // (self.L * self.N)
        out = torch.empty(tuple(x.shape[:-2]) + (self.dnum, self.D, self.N), dtype=x.dtype, device=x.device)
        self._check(load().ckks_modup(self.handle, _dev_ptr(x), _dev_ptr(out), batch, _stream()))
        return out

    def moddown(self, x: torch.Tensor) -> torch.Tensor:
        batch = x.numel() // (self.D * self.N)
        out = torch.empty(tuple(x.shape[:-2]) + (self.L, self.N), dtype=x.dtype, device=x.device)
        self._check(load().ckks_moddown(self.handle, _dev_ptr(x), _dev_ptr(out), batch, _stream()))
        return out

    def automorph(self, x: torch.Tensor, galois: int, eval_domain: bool, prime_first: int = 0) -> torch.Tensor:
        n_limbs = x.shape[-2]
        batch = x.numel() // (n_limbs * self.N)
        out = torch.empty_like(x)
        self._check(load().ckks_automorph(self.handle, _dev_ptr(x), _dev_ptr(out), prime_first, n_limbs, galois,
                                          1 if eval_domain else 0, batch, _stream()))
        return out

    def pointwise(self, op: int, a: torch.Tensor, b: torch.Tensor, out: Optional[torch.Tensor] = None,
                  prime_first: int = 0) -> torch.Tensor:
        """a (op) b limb by limb; a [..][n_limbs][N], b the same or fewer leading groups (applied cyclically).
        PW_MAC accumulates into `out`, which may be `a` or `b` for the other operations."""
        n_limbs = a.shape[-2]
        batch = a.numel() // (n_limbs * self.N)
        b_period = b.numel() // (n_limbs * self.N)
        if out is None:
            if op == PW_MAC:
                raise ValueError("PW_MAC accumulates into out")
            out = torch.empty_like(a)
        if b.shape[-2] != n_limbs or out.shape != a.shape:
            raise ValueError("operand shapes do not match")
        self._check(load().ckks_pointwise(self.handle, op, _dev_ptr(a), _dev_ptr(b), _dev_ptr(out), prime_first,
                                          n_limbs, batch, b_period, _stream()))
        return out

    def keyswitch(self, d: torch.Tensor, key: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        batch = d.numel() // (self.L * self.N)
        if out is None:
            out = torch.empty(tuple(d.shape[:-2]) + (2, self.L, self.N), dtype=d.dtype, device=d.device)
        ws = self.workspace(OP_KEYSWITCH, batch)
        self._check(load().ckks_keyswitch(self.handle, _dev_ptr(d), _dev_ptr(key), _dev_ptr(out), batch,
                                          ws.data_ptr(), ws.numel(), _stream()))
        return out

    def hmult_relin(self, ct1: torch.Tensor, ct2: torch.Tensor, evk: torch.Tensor,
                    out: Optional[torch.Tensor] = None) -> torch.Tensor:
        batch = ct1.numel() // (2 * self.L * self.N)
        if out is None:
            out = torch.empty_like(ct1)
        ws = self.workspace(OP_HMULT_RELIN, batch)
        self._check(load().ckks_hmult_relin(self.handle, _dev_ptr(ct1), _dev_ptr(ct2), _dev_ptr(evk), _dev_ptr(out),
                                            batch, ws.data_ptr(), ws.numel(), _stream()))
        return out

    def hrot(self, ct: torch.Tensor, galois: int, rk: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        batch = ct.numel() // (2 * self.L * self.N)
        if out is None:
            out = torch.empty_like(ct)
        ws = self.workspace(OP_HROT, batch)
        self._check(load().ckks_hrot(self.handle, _dev_ptr(ct), galois, _dev_ptr(rk), _dev_ptr(out), batch,
                                     ws.data_ptr(), ws.numel(), _stream()))
        return out

    def hrot_hoisted_mac(self, ct: torch.Tensor, galois: Sequence[int], rks: Sequence[torch.Tensor],
                         pt: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        n_rot = len(galois)
        if len(rks) != n_rot or pt.numel() != n_rot * self.L * self.N:
            raise ValueError("one key and one plaintext per rotation")
        if out is None:
            out = torch.empty_like(ct)
        g = (ctypes.c_uint32 * n_rot)(*[int(x) for x in galois])
        ptrs = (ctypes.c_void_p * n_rot)(*[_dev_ptr(k) for k in rks])
        ws = self.workspace(OP_HROT_HOISTED_MAC, n_rot)
        self._check(load().ckks_hrot_hoisted_mac(self.handle, _dev_ptr(ct), n_rot, ctypes.cast(g, _vp),
                                                 ctypes.cast(ptrs, _vp), _dev_ptr(pt), _dev_ptr(out),
                                                 ws.data_ptr(), ws.numel(), _stream()))
        return out

    # -- levels below L: tensors carry `level` limbs instead of L; keys stay full-level ----------
    def keyswitch_at(self, level: int, d: torch.Tensor, key: torch.Tensor,
                     out: Optional[torch.Tensor] = None) -> torch.Tensor:
        batch = d.numel() // (level * self.N)
        if out is None:
            out = torch.empty(tuple(d.shape[:-2]) + (2, level, self.N), dtype=d.dtype, device=d.device)
        ws = self.workspace(OP_KEYSWITCH, batch, level)
        self._check(load().ckks_keyswitch_at(self.handle, level, _dev_ptr(d), _dev_ptr(key), _dev_ptr(out), batch,
                                             ws.data_ptr(), ws.numel(), _stream()))
        return out

    def hmult_relin_at(self, level: int, ct1: torch.Tensor, ct2: torch.Tensor, evk: torch.Tensor,
                       out: Optional[torch.Tensor] = None) -> torch.Tensor:
        batch = ct1.numel() // (2 * level * self.N)
        if out is None:
            out = torch.empty_like(ct1)
        ws = self.workspace(OP_HMULT_RELIN, batch, level)
        self._check(load().ckks_hmult_relin_at(self.handle, level, _dev_ptr(ct1), _dev_ptr(ct2), _dev_ptr(evk),
                                               _dev_ptr(out), batch, ws.data_ptr(), ws.numel(), _stream()))
        return out

    def hrot_at(self, level: int, ct: torch.Tensor, galois: int, rk: torch.Tensor,
                out: Optional[torch.Tensor] = None) -> torch.Tensor:
        batch = ct.numel() // (2 * level * self.N)
        if out is None:
            out = torch.empty_like(ct)
        ws = self.workspace(OP_HROT, batch, level)
        self._check(load().ckks_hrot_at(self.handle, level, _dev_ptr(ct), galois, _dev_ptr(rk), _dev_ptr(out), batch,
                                        ws.data_ptr(), ws.numel(), _stream()))
        return out

    def hrot_hoisted_mac_at(self, level: int, ct: torch.Tensor, galois: Sequence[int], rks: Sequence[torch.Tensor],
                            pt: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        n_rot = len(galois)
        if len(rks) != n_rot or pt.numel() != n_rot * level * self.N:
            raise ValueError("one key and one plaintext per rotation")
        if out is None:
            out = torch.empty_like(ct)
        g = (ctypes.c_uint32 * n_rot)(*[int(x) for x in galois])
        ptrs = (ctypes.c_void_p * n_rot)(*[_dev_ptr(k) for k in rks])
        ws = self.workspace(OP_HROT_HOISTED_MAC, n_rot, level)
        self._check(load().ckks_hrot_hoisted_mac_at(self.handle, level, _dev_ptr(ct), n_rot, ctypes.cast(g, _vp),
                                                    ctypes.cast(ptrs, _vp), _dev_ptr(pt), _dev_ptr(out),
                                                    ws.data_ptr(), ws.numel(), _stream()))
        return out

    def rescale(self, level: int, ct: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """ct [batch...][2][level][N] -> [batch...][2][level-1][N]."""
        batch = ct.numel() // (2 * level * self.N)
        if out is None:
            out = torch.empty(tuple(ct.shape[:-2]) + (level - 1, self.N), dtype=ct.dtype, device=ct.device)
        ws = self.workspace(OP_RESCALE, batch, level)
        self._check(load().ckks_rescale(self.handle, level, _dev_ptr(ct), _dev_ptr(out), batch,
                                        ws.data_ptr(), ws.numel(), _stream()))
        return out

    def hrot_dh_mac(self, ct: torch.Tensor, galois: Sequence[int], rks: Sequence[torch.Tensor], pt: torch.Tensor,
                    out: Optional[torch.Tensor] = None, level: Optional[int] = None) -> torch.Tensor:
        """Double-hoisted rotate-MAC; pt [n_rot][level+K][N] on the level's extended basis."""
        ell = self.L if level is None else level
        n_rot = len(galois)
        if len(rks) != n_rot or pt.numel() != n_rot * (ell + self.K) * self.N:
            raise ValueError("one key and one extended-basis plaintext per rotation")
        if out is None:
            out = torch.empty_like(ct)
        g = (ctypes.c_uint32 * n_rot)(*[int(x) for x in galois])
        ptrs = (ctypes.c_void_p * n_rot)(*[_dev_ptr(k) for k in rks])
        ws = self.workspace(OP_HROT_DH_MAC, n_rot, ell)
        if level is None:
            rc = load().ckks_hrot_dh_mac(self.handle, _dev_ptr(ct), n_rot, ctypes.cast(g, _vp), ctypes.cast(ptrs, _vp),
                                         _dev_ptr(pt), _dev_ptr(out), ws.data_ptr(), ws.numel(), _stream())
        else:
            rc = load().ckks_hrot_dh_mac_at(self.handle, ell, _dev_ptr(ct), n_rot, ctypes.cast(g, _vp),
                                            ctypes.cast(ptrs, _vp), _dev_ptr(pt), _dev_ptr(out), ws.data_ptr(),
                                            ws.numel(), _stream())
        self._check(rc)
        return out

    # -- ModDown merged with the following rescale: outputs carry level - 1 limbs -----------------
    def hmult_relin_rescale_at(self, level: int, ct1: torch.Tensor, ct2: torch.Tensor, evk: torch.Tensor,
                               out: Optional[torch.Tensor] = None) -> torch.Tensor:
        batch = ct1.numel() // (2 * level * self.N)
        if out is None:
            out = torch.empty(tuple(ct1.shape[:-2]) + (level - 1, self.N), dtype=ct1.dtype, device=ct1.device)
        ws = self.workspace(OP_HMULT_RELIN, batch, level)
        self._check(load().ckks_hmult_relin_rescale_at(self.handle, level, _dev_ptr(ct1), _dev_ptr(ct2), _dev_ptr(evk),
                                                       _dev_ptr(out), batch, ws.data_ptr(), ws.numel(), _stream()))
        return out

    def hrot_dh_mac_rescale_at(self, level: int, ct: torch.Tensor, galois: Sequence[int], rks: Sequence[torch.Tensor],
                               pt: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        n_rot = len(galois)
        if len(rks) != n_rot or pt.numel() != n_rot * (level + self.K) * self.N:
            raise ValueError("one key and one extended-basis plaintext per rotation")
        if out is None:
            out = torch.empty((2, level - 1, self.N), dtype=ct.dtype, device=ct.device)
        g = (ctypes.c_uint32 * n_rot)(*[int(x) for x in galois])
        ptrs = (ctypes.c_void_p * n_rot)(*[_dev_ptr(k) for k in rks])
        ws = self.workspace(OP_HROT_DH_MAC, n_rot, level)
        self._check(load().ckks_hrot_dh_mac_rescale_at(self.handle, level, _dev_ptr(ct), n_rot, ctypes.cast(g, _vp),
                                                       ctypes.cast(ptrs, _vp), _dev_ptr(pt), _dev_ptr(out),
                                                       ws.data_ptr(), ws.numel(), _stream()))
        return out

    def lintrans_bsgs_at(self, level: int, ct: torch.Tensor, baby_galois: Sequence[int], baby_rks: Sequence[torch.Tensor],
                         giant_galois: Sequence[int], giant_rks: Sequence[torch.Tensor], pt: torch.Tensor,
                         out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """pt [n2][n1][level+K][N]; out = sum_g HRot_g(sum_b pt[g][b] * HRot_b(ct)), baby steps double-hoisted."""
        n1, n2 = len(baby_galois), len(giant_galois)
        if len(baby_rks) != n1 or len(giant_rks) != n2 or pt.numel() != n1 * n2 * (level + self.K) * self.N:
            raise ValueError("one key per rotation and one extended-basis plaintext per (giant, baby) pair")
        if out is None:
            out = torch.empty_like(ct)
        need = _sz()
        self._check(load().ckks_lintrans_bsgs_workspace_bytes(self.handle, level, n1, n2, ctypes.byref(need)))
        if self._ws is None or self._ws.numel() < need.value:
            self._ws = None
            self._ws = torch.empty(need.value, dtype=torch.uint8, device=self.device)
        bg = (ctypes.c_uint32 * n1)(*[int(x) for x in baby_galois])
        gg = (ctypes.c_uint32 * n2)(*[int(x) for x in giant_galois])
        bk = (ctypes.c_void_p * n1)(*[_dev_ptr(k) for k in baby_rks])
        gk = (ctypes.c_void_p * n2)(*[_dev_ptr(k) for k in giant_rks])
        self._check(load().ckks_lintrans_bsgs_at(self.handle, level, _dev_ptr(ct), n1, ctypes.cast(bg, _vp),
                                                 ctypes.cast(bk, _vp), n2, ctypes.cast(gg, _vp), ctypes.cast(gk, _vp),
                                                 _dev_ptr(pt), _dev_ptr(out), self._ws.data_ptr(), self._ws.numel(),
                                                 _stream()))
        return out

    def hrot_multi_at(self, level: int, ct: torch.Tensor, galois: Sequence[int], rks: Sequence[torch.Tensor],
                      out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """ct [batch][2][level][N]; instance b is rotated by galois[b] with key rks[b]."""
        batch = len(galois)
        if len(rks) != batch or ct.numel() != batch * 2 * level * self.N:
            raise ValueError("one Galois element and one key per ciphertext")
        if out is None:
            out = torch.empty_like(ct)
        g = (ctypes.c_uint32 * batch)(*[int(x) for x in galois])
        ptrs = (ctypes.c_void_p * batch)(*[_dev_ptr(k) for k in rks])
        ws = self.workspace(OP_HROT, min(batch, ROTATIONS_PER_LAUNCH), level)
        self._check(load().ckks_hrot_multi_at(self.handle, level, _dev_ptr(ct), ctypes.cast(g, _vp), ctypes.cast(ptrs, _vp),
                                              _dev_ptr(out), batch, ws.data_ptr(), ws.numel(), _stream()))
        return out
