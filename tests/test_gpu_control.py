"""GPU parity, integer work (bit-exact): active-set compaction, UpdateMASK, lock rule."""
import numpy as np
import pytest
import torch

from oracle import control
from paper_2602_06412_amd import binding as B
from tests.gpu_util import DEV, compact, dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("Bn,N,p", [(1, 1, 0.5), (1, 128, 0.3), (3, 100, 0.7), (8, 1024, 0.5),
                                    (2, 2053, 0.9), (1, 2048, 0.0), (4, 777, 1.0), (8, 8192, 0.25)])
def test_compact_active(Bn, N, p):
    rng = np.random.default_rng(Bn * 100003 + N)
    lock = (rng.random((Bn, N)) < p).astype(np.uint8)
    idx, cu = compact(lock)
    want_idx, want_cu = control.compact_active(lock)
    assert np.array_equal(cu, want_cu)
    assert np.array_equal(idx, want_idx)


def _unmask_case(rng, Bn, N, lo, hi, k, ties):
    lock = (rng.random((Bn, N)) < 0.3).astype(np.uint8)
    masked = ((rng.random((Bn, N)) < 0.6) & (lock == 0)).astype(np.uint8)
    idx, cu = control.compact_active(lock)
    M = len(idx)
    conf = rng.random(M).astype(np.float32)
    if ties:
        conf = (np.floor(conf * 4) / 4).astype(np.float32)
    amax = rng.integers(0, 50000, M).astype(np.int32)
    tokens = rng.integers(0, 50000, (Bn, N)).astype(np.int32)
    # oracle, sequence by sequence
    want_tok, want_msk = tokens.copy(), masked.copy()
    for b in range(Bn):
        r0, r1 = cu[b], cu[b + 1]
        control.update_mask(want_msk[b], want_tok[b], idx[r0:r1] - b * N, conf[r0:r1], amax[r0:r1], lo, hi, k)
    t_tok, t_msk = dev(tokens.reshape(-1)), dev(masked.reshape(-1))
    B.sl_unmask_topk(t_tok, t_msk, dev(idx, torch.int32), dev(cu, torch.int32), dev(conf), dev(amax), Bn, N, lo, hi, k)
    torch.cuda.synchronize()
    assert np.array_equal(t_tok.cpu().numpy().reshape(Bn, N), want_tok)
    assert np.array_equal(t_msk.cpu().numpy().reshape(Bn, N), want_msk)


@pytest.mark.parametrize("Bn,N,lo,hi,k,ties", [(1, 128, 32, 128, 3, False), (1, 128, 32, 128, 3, True),
                                               (8, 1024, 512, 1024, 1, False), (3, 300, 37, 101, 7, True),
                                               (2, 2048, 1024, 1088, 64, True), (1, 64, 10, 20, 100, False),
                                               (2, 50, 5, 5, 3, False), (2, 50, 0, 50, 0, False)])
def test_unmask_topk(Bn, N, lo, hi, k, ties):
    _unmask_case(np.random.default_rng(N * 7 + k), Bn, N, lo, hi, k, ties)


@pytest.mark.parametrize("Bn,N,first", [(1, 128, 0), (1, 128, 1), (8, 1024, 0), (3, 333, 0)])
def test_lock_rule(Bn, N, first):
    rng = np.random.default_rng(N + first)
    lock = (rng.random((Bn, N)) < 0.4).astype(np.uint8)
    masked = ((rng.random((Bn, N)) < 0.5) & (lock == 0)).astype(np.uint8)
    idx, cu = control.compact_active(lock)
    M = len(idx)
    kl = rng.random(M).astype(np.float32)
    kl[rng.random(M) < 0.1] = np.inf
    eps = rng.random(Bn).astype(np.float32)
    if M:
        eps[idx[0] // N] = kl[0]                       # exact equality must lock (<=)
    want = lock.copy()
    for b in range(Bn):
        r0, r1 = cu[b], cu[b + 1]
        F = control.lock_rule(lock[b], masked[b], idx[r0:r1] - b * N, kl[r0:r1], np.zeros(r1 - r0), eps[b], bool(first))
        want[b, F] = 1
    for alias in (False, True):
        t_lock = dev(lock.reshape(-1))
        out = t_lock if alias else torch.full((Bn * N,), 7, dtype=torch.uint8, device=DEV)
        B.sl_lock_rule(t_lock, dev(masked.reshape(-1)), dev(idx, torch.int32), dev(cu, torch.int32)[Bn:], Bn * N,
                       dev(kl), dev(eps), Bn, N, first, out)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy().reshape(Bn, N), want)


def test_empty_active_set():
    lock = np.ones((2, 64), dtype=np.uint8)
    idx, cu = compact(lock)
    assert len(idx) == 0 and list(cu) == [0, 0, 0]


@pytest.mark.parametrize("Bn,N,m,first,ties,p_masked", [
    (1, 128, 20.0, 0, False, 0.5), (1, 128, 20.0, 1, False, 0.5), (8, 1024, 20.0, 0, False, 0.5),
    (3, 333, 50.0, 0, True, 0.3), (2, 2048, 100.0, 0, False, 0.1), (4, 777, 0.5, 0, True, 0.6),
    (2, 64, 33.3, 0, True, 0.0), (3, 100, 20.0, 0, False, 1.0), (1, 15360, 7.0, 0, False, 0.2)])
def test_lock_rule_with_confidence_gate(Bn, N, m, first, ties, p_masked):
    """The gated lock rule (nearest-rank percentile of u over the candidates of each sequence)
    against the oracle's, on the same fp32 inputs: bit-exact masks.  Covers ties at the threshold,
    an empty candidate set (everything masked), m = 100 and a first step."""
    rng = np.random.default_rng(N * 31 + int(m * 10) + first)
    lock = (rng.random((Bn, N)) < 0.4).astype(np.uint8)
    masked = ((rng.random((Bn, N)) < p_masked) & (lock == 0)).astype(np.uint8)
    idx, cu = control.compact_active(lock)
    M = len(idx)
    conf = rng.random(M).astype(np.float32)
    if ties:
        conf = (np.floor(conf * 8) / 8).astype(np.float32)
    conf[rng.random(M) < 0.02] = np.float32(1.0000001)          # rounding can push a confidence past 1
    kl = (rng.random(M) * 2e-3).astype(np.float32)
    eps = (rng.random(Bn) * 2e-3).astype(np.float32)
    m32 = np.float32(m)
    u = np.maximum(np.float32(0), np.float32(1) - conf).astype(np.float32)
    want = lock.copy()
    for b in range(Bn):
        r0, r1 = cu[b], cu[b + 1]
        F = control.lock_rule(lock[b], masked[b], idx[r0:r1] - b * N, kl[r0:r1], u[r0:r1], eps[b], bool(first),
                              gate_m=float(m32))
        want[b, F] = 1
    out = torch.full((Bn * N,), 7, dtype=torch.uint8, device=DEV)
    B.sl_lock_rule_gated(dev(lock.reshape(-1)), dev(masked.reshape(-1)), dev(idx, torch.int32), dev(cu, torch.int32), M,
                         dev(kl), dev(conf), dev(eps), float(m32), Bn, N, first, out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy().reshape(Bn, N), want)
    if not first and p_masked < 1.0:
        assert want.sum() > lock.sum(), "the case should lock something"


def test_lock_rule_gated_argument_errors():
    z8 = torch.zeros(8, dtype=torch.uint8, device=DEV)
    zi = torch.zeros(8, dtype=torch.int32, device=DEV)
    zf = torch.zeros(8, device=DEV)
    for bad_m in (0.0, -1.0, 100.5):
        with pytest.raises(B.SureLockError):
            B.sl_lock_rule_gated(z8, z8, zi, zi, 4, zf, zf, zf, bad_m, 1, 8, 0, z8)
    with pytest.raises(B.SureLockError):
        B.sl_lock_rule_gated(z8, z8, zi, zi, 4, zf, zf, zf, 20.0, 1, 20000, 0, z8)      # n_seq beyond the LDS budget
