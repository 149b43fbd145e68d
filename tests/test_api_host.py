"""Host-only checks of the C ABI: the built library loads, exports every symbol the header
declares, and rejects bad arguments before touching the GPU."""
import ctypes
import os
import re

import pytest

from paper_2310_16530_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2310_16530_amd import binding, build
    if build.is_stale():
        build.build()
    return binding.load()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "ckks_mi355x.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ckks_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    from paper_2310_16530_amd import binding
    names = declared_symbols()
    assert "ckks_keyswitch" in names and "ckks_hrot_hoisted_mac" in names and len(names) >= 15
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names


def test_table_bytes_and_shape_validation(lib):
    n = ctypes.c_size_t()
    assert lib.ckks_table_bytes(16, 24, 6, 4, ctypes.byref(n)) == 0
    # 30 primes x (4 integer + 2 floating-point) twiddle tables x 2^16 words dominate
    assert 30 * 6 * 65536 * 8 <= n.value <= 30 * 6 * 65536 * 8 + (1 << 20)
    assert lib.ckks_table_bytes(16, 24, 6, 4, None) == -1
    assert lib.ckks_table_bytes(11, 24, 6, 4, ctypes.byref(n)) == -2      # ring too small
    assert lib.ckks_table_bytes(17, 24, 6, 4, ctypes.byref(n)) == -2      # ring too large
    assert lib.ckks_table_bytes(16, 24, 6, 5, ctypes.byref(n)) == 0       # digits of 5, 5, 5, 5, 4 limbs
    assert lib.ckks_table_bytes(16, 9, 3, 4, ctypes.byref(n)) == -2       # digits of 3 limbs make 3 digits, not 4
    assert lib.ckks_table_bytes(16, 3, 3, 4, ctypes.byref(n)) == -1       # more digits than limbs
    assert lib.ckks_table_bytes(16, 0, 6, 1, ctypes.byref(n)) == -1
    assert lib.ckks_table_bytes(16, 24, 6, 0, ctypes.byref(n)) == -1
    assert lib.ckks_table_bytes(16, 60, 15, 4, ctypes.byref(n)) == 0      # L = 60 in four digits of 15 limbs
    assert lib.ckks_table_bytes(16, 120, 9, 8, ctypes.byref(n)) == -2     # too many primes
    assert lib.ckks_table_bytes(16, 24, 17, 4, ctypes.byref(n)) == -2     # K too large
    assert lib.ckks_table_bytes(16, 34, 3, 2, ctypes.byref(n)) == -2      # alpha = 17 too large
    assert lib.ckks_table_bytes(16, 32, 16, 2, ctypes.byref(n)) == 0      # the widest digits
    assert lib.ckks_table_bytes(16, 24, 0, 1, ctypes.byref(n)) == 0       # transform-only context


def test_ctx_create_rejects_bad_arguments_on_the_host(lib):
    ps = synth.CFG0
    pr = (ctypes.c_uint64 * 4)(*ps.primes)
    h = ctypes.c_void_p()
    fake = ctypes.c_void_p(1 << 20)   # never dereferenced: every case below fails before the copy
    big = 1 << 30
    assert lib.ckks_ctx_create(None, 12, 3, 1, 3, pr, None, fake, big, None) == -1
    assert lib.ckks_ctx_create(ctypes.byref(h), 12, 3, 1, 3, None, None, fake, big, None) == -1
    assert lib.ckks_ctx_create(ctypes.byref(h), 12, 3, 1, 3, pr, None, None, big, None) == -1
    assert lib.ckks_ctx_create(ctypes.byref(h), 12, 3, 1, 3, pr, None, ctypes.c_void_p((1 << 20) + 8), big, None) == -1
    assert lib.ckks_ctx_create(ctypes.byref(h), 12, 3, 1, 3, pr, None, fake, 1024, None) == -4
    assert lib.ckks_ctx_create(ctypes.byref(h), 11, 3, 1, 3, pr, None, fake, big, None) == -2   # ring too small
    assert lib.ckks_ctx_create(ctypes.byref(h), 12, 3, 1, 4, pr, None, fake, big, None) == -1   # more digits than limbs
    bad = (ctypes.c_uint64 * 4)(ps.primes[0], ps.primes[1], ps.primes[1], ps.primes[3])      # duplicate
    assert lib.ckks_ctx_create(ctypes.byref(h), 12, 3, 1, 3, bad, None, fake, big, None) == -1
    bad = (ctypes.c_uint64 * 4)(ps.primes[0], ps.primes[1], ps.primes[2] + 2 * 8192, ps.primes[3])  # composite
    assert not synth.is_prime(ps.primes[2] + 2 * 8192)
    assert lib.ckks_ctx_create(ctypes.byref(h), 12, 3, 1, 3, bad, None, fake, big, None) == -1
    bad = (ctypes.c_uint64 * 4)(ps.primes[0], ps.primes[1], 1000003, ps.primes[3])           # not 1 mod 2N
    assert lib.ckks_ctx_create(ctypes.byref(h), 12, 3, 1, 3, bad, None, fake, big, None) == -1
    bad = (ctypes.c_uint64 * 4)(ps.primes[0], ps.primes[1], ps.primes[2], (1 << 61) + 20 * 8192 + 1)  # too wide
    assert lib.ckks_ctx_create(ctypes.byref(h), 12, 3, 1, 3, bad, None, fake, big, None) in (-1, -2)
    psi = (ctypes.c_uint64 * 4)(2, 3, 5, 7)                                                  # not 2N-th roots
    assert lib.ckks_ctx_create(ctypes.byref(h), 12, 3, 1, 3, pr, psi, fake, big, None) == -1
    assert not h.value


def test_null_context_calls_fail_cleanly(lib):
    fake = ctypes.c_void_p(1 << 20)
    n = ctypes.c_size_t()
    assert lib.ckks_ntt(None, fake, 0, 1, 1, None) == -1
    assert lib.ckks_intt(None, fake, 0, 1, 1, None) == -1
    assert lib.ckks_modup(None, fake, fake, 1, None) == -1
    assert lib.ckks_moddown(None, fake, fake, 1, None) == -1
    assert lib.ckks_automorph(None, fake, fake, 0, 1, 5, 1, 1, None) == -1
    assert lib.ckks_keyswitch(None, fake, fake, fake, 1, fake, 0, None) == -1
    assert lib.ckks_hmult_relin(None, fake, fake, fake, fake, 1, fake, 0, None) == -1
    assert lib.ckks_hrot(None, fake, 5, fake, fake, 1, fake, 0, None) == -1
    assert lib.ckks_hrot_hoisted_mac(None, fake, 1, fake, fake, fake, fake, fake, 0, None) == -1
    assert lib.ckks_workspace_bytes(None, 4, 1, ctypes.byref(n)) == -1
    assert lib.ckks_profile_enable(None, 1) == -1
    assert lib.ckks_set_overlap(None, 1) == -1
    assert lib.ckks_last_error(None) == b"null context"
    assert lib.ckks_ctx_psi(None, 0) == 0
    lib.ckks_ctx_destroy(None)


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr


def test_binding_operand_checks_reject_before_any_launch():
    """The binding checks what the C ABI cannot see (buffer lengths, dtype, layout, device); the checks run on
    the host, so CPU tensors exercise every branch: a wrong size is reported before the device is looked at."""
    import torch
    from paper_2310_16530_amd import binding
    N, L, K, dnum = 4096, 3, 1, 3
    good = torch.zeros((2, L, N), dtype=torch.int64)
    with pytest.raises(ValueError, match="64-bit"):
        binding.check_operand(torch.zeros(8, dtype=torch.int32), 8, "x")
    with pytest.raises(ValueError, match="64-bit"):
        binding.check_operand(torch.zeros(8, dtype=torch.float64), 8, "x")
    with pytest.raises(ValueError, match="contiguous"):
        binding.check_operand(good.transpose(0, 1), good.numel(), "ct")
    with pytest.raises(ValueError, match="expected"):
        binding.check_operand(good, good.numel() - N, "ct")            # one limb short
    with pytest.raises(ValueError, match="expected"):
        binding.check_operand(torch.zeros((dnum, 2, L, N), dtype=torch.int64), dnum * 2 * (L + K) * N, "key")  # key without special limbs
    with pytest.raises(ValueError, match="is on cpu"):
        binding.check_operand(good, good.numel(), "ct", torch.device("cuda:0"))   # right size, wrong device
    assert binding.check_batch(good, L * N, "x") == 2
    with pytest.raises(ValueError, match="multiple"):
        binding.check_batch(good, 4 * N, "x")
    with pytest.raises(ValueError, match="multiple"):
        binding.check_batch(torch.zeros(0, dtype=torch.int64), N, "x")
    with pytest.raises(ValueError, match="primes"):
        binding.check_chain(3, 1, synth.CFG0.primes[:3], None)
    with pytest.raises(ValueError, match="roots"):
        binding.check_chain(3, 1, synth.CFG0.primes, [1, 2, 3])
    with pytest.raises(ValueError, match="primes"):
        binding.Context(12, 3, 1, 3, synth.CFG0.primes[:3])          # rejected before the library is touched
    binding.check_chain(3, 1, synth.CFG0.primes, None)
