"""The entry point that allocates nothing: ckks_rescale_static against ckks_rescale through the C ABI
(needs an MI355X).  Integer work: the two must agree word for word.  Two calls in a row share the GPU's static
scratch array, the second with a smaller input, so stale contents of the first call must not leak into it."""
import ctypes

import numpy as np
import pytest

from paper_2310_16530_amd import synth

pytestmark = pytest.mark.gpu


def test_rescale_static_matches_rescale_on_two_calls_in_a_row():
    import torch
    from paper_2310_16530_amd import binding
    lib = binding.load()
    ps = synth.small_params(14, 6, 2, 3)
    ctx = binding.Context(ps.logN, ps.L, ps.K, ps.dnum, ps.primes)
    h = ctx.handle
    rng = np.random.default_rng(2024)

    def run(level, batch):
        print("rescale_static: level", level, "batch", batch, flush=True)
        ct = synth.uniform_residues(rng, ps.q_primes[:level], ps.N, lead=(batch, 2))
        d_ct = torch.from_numpy(ct.view(np.int64)).to("cuda:0")
        ws = ctx.workspace(binding.OP_RESCALE, batch, level)
        want = torch.empty((batch, 2, level - 1, ps.N), dtype=torch.int64, device="cuda:0")
        got = torch.full_like(want, -1)
        stream = torch.cuda.current_stream().cuda_stream
        assert lib.ckks_rescale(h, level, d_ct.data_ptr(), want.data_ptr(), batch, ws.data_ptr(), ws.numel(), stream) == 0
        assert lib.ckks_rescale_static(h, level, d_ct.data_ptr(), got.data_ptr(), batch, stream) == 0
        torch.cuda.synchronize()
        assert torch.equal(got, want), (level, batch)

    run(6, 3)      # 3 ciphertexts at the top level: 36 limbs of scratch
    run(4, 1)      # then a smaller input: 8 limbs, the rest of the scratch still holds the first call's words
    run(6, 3)
    # beyond the static array: rejected with a clear error, nothing launched
    big = ctypes.c_void_p(1 << 30)   # never dereferenced
    n_max = binding.STATIC_SCRATCH_BYTES // (2 * 6 * ps.N * 8)
    assert lib.ckks_rescale_static(h, 6, big, ctypes.c_void_p((1 << 30) + (1 << 29)), n_max + 1, None) == binding.CKKS_ENOMEM
    assert b"CKKS_STATIC_SCRATCH_BYTES" in lib.ckks_last_error(h)
    assert lib.ckks_rescale_static(h, 1, big, big, 1, None) == binding.CKKS_EINVAL
    assert lib.ckks_rescale_static(None, 2, big, big, 1, None) == binding.CKKS_EINVAL
    torch.cuda.synchronize()
