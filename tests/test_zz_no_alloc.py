"""sl_sample_tokens_noalloc (the token draw for callers that cannot allocate: its per-part candidates
live in a buffer inside the library's device code) against sl_sample_tokens with a caller's scratch:
bit-identical drawn ids on two calls in a row, the second on a smaller input, so that whatever the
first call left in the shared buffer must not leak into the second; and the size limit is an error."""
import numpy as np
import pytest
import torch

from oracle import control
from paper_2602_06412_amd import binding as B
from tests.gpu_util import DEV, dev

pytestmark = pytest.mark.gpu


def _case(seed, T, V, Bn, N, tau, packed):
    rng = np.random.default_rng(seed)
    lock = (rng.random((Bn, N)) < 0.3).astype(np.uint8)
    masked = ((rng.random((Bn, N)) < 0.7) & (lock == 0)).astype(np.uint8)
    idx, cu = control.compact_active(lock)
    M = len(idx)
    z = (torch.randn(M if packed else Bn * N, V, generator=torch.Generator().manual_seed(seed)) * 2.0).to(T).to(DEV)
    argmax = dev(rng.integers(0, V, M).astype(np.int32))
    args = (z, packed, B.dtype_code(T), V, dev(idx, torch.int32), dev(cu, torch.int32)[Bn:], M, dev(masked.reshape(-1)), N,
            N // 8, N - N // 8, tau, 0x0123456789abcdef + seed, 3 + seed, argmax)
    pos = idx % N
    n_elig = int(((masked.reshape(-1)[idx] == 1) & (pos >= N // 8) & (pos < N - N // 8)).sum())
    return args, M, n_elig


def test_noalloc_draw_equals_the_scratch_argument_form_twice_in_a_row():
    # second call: fewer rows, another vocabulary and dtype, so stale candidates of the first call sit in the buffer
    for seed, T, V, Bn, N, tau, packed in ((1, torch.bfloat16, 126464, 2, 160, 1.0, 0), (2, torch.float32, 4160, 1, 48, 0.6, 1)):
        args, M, n_elig = _case(seed, T, V, Bn, N, tau, packed)
        assert n_elig > 8
        want = torch.full((M,), -7, dtype=torch.int32, device=DEV)
        got = torch.full((M,), -9, dtype=torch.int32, device=DEV)
        B.sl_sample_tokens(*args, want)
        B.sl_sample_tokens_noalloc(*args, got)
        torch.cuda.synchronize()
        assert torch.equal(got, want), f"case {seed}"
        assert int((want != args[-1]).sum().item()) >= n_elig // 2      # draws did happen


def test_noalloc_draw_rejects_sizes_beyond_its_buffer():
    args, M, _ = _case(3, torch.float32, 64, 1, 32, 1.0, 1)
    out = torch.zeros(M, dtype=torch.int32, device=DEV)
    a = list(args)
    a[6] = 16385                                        # m_upper beyond the static buffer's 16384 rows
    with pytest.raises(B.SureLockError) as e:
        B.sl_sample_tokens_noalloc(*a, out)
    assert e.value.status == B.SL_ENOSPC
    a[6] = M
    B.sl_sample_tokens_noalloc(*a, out)                 # and the library still works afterwards
    torch.cuda.synchronize()
