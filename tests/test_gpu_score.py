"""GPU parity of the posterior scoring kernel (step-wise KL, confidence, argmax) against the
oracle's fp64 definitions.  Tolerance on KL: 1e-4 relative plus 2e-7 absolute (the fp32
floor of a difference of two logsumexps of O(10) magnitude is ~1e-6; the kernel's
difference form keeps it well below that)."""
import numpy as np
import pytest
import torch

from oracle import posterior, rounding
from paper_2602_06412_amd import binding as B
from tests.gpu_util import DEV, dev

pytestmark = pytest.mark.gpu

KL_RTOL, KL_ATOL = 1e-4, 2e-7


def _rows(seed, R, V, storage, scale, delta):
    rng = np.random.default_rng(seed)
    rnd = rounding.STORAGE[storage]
    z0 = rnd(rng.standard_normal((R, V)) * scale)
    z1 = rnd(z0 + delta * rng.standard_normal((R, V)))
    return z0, z1


def _run(z_prev, z_cur, storage, active, packed, first=False):
    T = {"fp32": torch.float32, "bf16": torch.bfloat16}[storage]
    R, V = z_prev.shape
    M = len(active)
    cur_np = z_cur[active] if packed else z_cur
    cur, prev = dev(cur_np, T), dev(z_prev, T)
    kl = torch.full((M + 3,), -7.0, device=DEV)
    conf = torch.full((M + 3,), -7.0, device=DEV)
    am = torch.full((M + 3,), -7, dtype=torch.int32, device=DEV)
    m_dev = dev(np.array([M], dtype=np.int32))
    B.sl_score_posteriors(cur, packed, prev, B.dtype_code(T), V, dev(active, torch.int32), m_dev, M + 3, first,
                          kl, conf, am)
    torch.cuda.synchronize()
    # rows beyond the true M must not be touched
    assert torch.all(kl[M:] == -7.0) and torch.all(am[M:] == -7)
    return kl[:M].cpu().numpy().astype(np.float64), conf[:M].cpu().numpy().astype(np.float64), am[:M].cpu().numpy()


@pytest.mark.parametrize("storage,V,scale,delta", [
    ("fp32", 1024, 0.3, 0.05), ("fp32", 1024, 3.0, 1.0), ("bf16", 4160, 1.3, 0.02), ("bf16", 126464, 1.3, 0.05),
    ("bf16", 126464, 1.3, 0.0), ("bf16", 126464, 6.0, 2.0), ("fp32", 126464, 1.3, 1e-3), ("bf16", 8, 2.0, 0.5)])
@pytest.mark.parametrize("packed", [0, 1])
def test_score_matches_oracle(storage, V, scale, delta, packed):
    R = 12
    z0, z1 = _rows(V + int(scale * 10), R, V, storage, scale, delta)
    active = np.array([0, 2, 3, 7, 11])
    kl, conf, am = _run(z0, z1, storage, active, packed)
    lp1, lp0 = posterior.log_softmax(z1[active]), posterior.log_softmax(z0[active])
    want_kl = posterior.kl_rows(lp1, lp0)
    assert np.all(np.abs(kl - want_kl) <= KL_RTOL * want_kl + KL_ATOL), (kl, want_kl)
    assert np.allclose(conf, posterior.max_prob(lp1), rtol=2e-6, atol=0)
    assert np.array_equal(am, posterior.argmax_lowest(z1[active]))
    assert np.all(kl >= 0)
    if delta == 0.0:
        assert np.all(kl == 0.0)                              # KL(p || p) = 0 exactly


def test_score_peaked_posteriors_and_pinsker():
    # one dominant token (a trained model's converged slot), small drift between steps
    V, R = 126464, 6
    rng = np.random.default_rng(5)
    z0 = rounding.round_bf16(rng.standard_normal((R, V)))
    z0[np.arange(R), rng.integers(0, V, R)] = 17.0
    z1 = rounding.round_bf16(z0 + 0.01 * rng.standard_normal((R, V)))
    active = np.arange(R)
    kl, conf, am = _run(z0, z1, "bf16", active, 0)
    lp1, lp0 = posterior.log_softmax(z1), posterior.log_softmax(z0)
    want = posterior.kl_rows(lp1, lp0)
    assert np.all(np.abs(kl - want) <= KL_RTOL * want + KL_ATOL), (kl, want)
    l1 = np.abs(np.exp(lp1) - np.exp(lp0)).sum(-1)
    assert np.all(l1 <= np.sqrt(2 * kl) + 1e-4)               # Pinsker with the GPU's KL
    assert np.allclose(1 - conf, posterior.uncertainty(lp1), rtol=0, atol=1e-6)


def test_score_first_step_and_argmax_ties():
    V = 4160
    z = np.zeros((4, V))
    z[0, [5, 9, 4000]] = 2.0                                   # three-way tie -> lowest id
    z[1, :] = -1.5                                             # all equal -> id 0
    z[2, V - 1] = 3.0
    z[3, [4159, 17]] = 1.0
    kl, conf, am = _run(z, z, "bf16", np.arange(4), 0, first=True)
    assert np.all(np.isinf(kl)) and np.all(kl > 0)
    assert list(am) == [5, 0, V - 1, 17]
    assert np.allclose(conf, posterior.max_prob(posterior.log_softmax(z)), rtol=2e-6)


def test_score_large_shift_between_rows():
    # previous row's maximum far above the current one's (an unmasking event): no overflow
    V = 1024
    rng = np.random.default_rng(9)
    z0 = rng.standard_normal((3, V)); z0[:, 3] = 40.0
    z1 = rng.standard_normal((3, V)); z1[:, 7] = -30.0
    z0, z1 = rounding.round_f32(z0), rounding.round_f32(z1)
    kl, conf, am = _run(z0, z1, "fp32", np.arange(3), 0)
    want = posterior.kl_rows(posterior.log_softmax(z1), posterior.log_softmax(z0))
    assert np.all(np.isfinite(kl)) and np.allclose(kl, want, rtol=1e-4)


def test_score_nan_row_gives_valid_argmax():
    """A row without a single comparable logit (all NaN) must still yield a token id inside the
    vocabulary: the id is written into `tokens` by UpdateMASK and indexes the embedding table in
    the next step.  Finite rows beside it are unaffected."""
    V, R = 4160, 3
    z0, z1 = _rows(7, R, V, "fp32", 1.0, 0.1)
    z1n = z1.copy()
    z1n[1, :] = np.nan
    _, _, am = _run(z0, z1n, "fp32", np.arange(R), packed=False)
    assert 0 <= am[1] < V
    assert am[0] == int(np.argmax(z1[0])) and am[2] == int(np.argmax(z1[2]))
