"""Pins of the oracle's arithmetic against things other than itself: closed forms,
hand-worked values, brute-force loops, and library routines used only as
independent third opinions (never as the oracle)."""
import itertools
import math

import numpy as np
import pytest
import scipy.special
import torch

from oracle import model, posterior, rounding


# ---------------------------------------------------------------- rounding
def test_round_bf16_matches_torch_on_fp32_inputs():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000) * s for s in (1e-3, 1.0, 37.0, 1e4)]).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    got = rounding.round_bf16(x.astype(np.float64))
    assert np.array_equal(got, want)


def test_round_bf16_ties_to_even_and_single_rounding():
    # bf16 neighbours of 1.0 are 1.0 and 1+2^-7; the midpoint ties to the even one (1.0)
    assert rounding.round_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    # next midpoint (between 1+2^-7 and 1+2^-6) ties up to the even 1+2^-6
    assert rounding.round_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    # just above a midpoint by less than an fp32 ulp must round up (a double
    # rounding through fp32 would land on the tie and go down)
    assert rounding.round_bf16(np.array([1.0 + 2.0 ** -8 + 2.0 ** -40]))[0] == 1.0 + 2.0 ** -7
    x = np.array([-3.3, 0.0, 1e-3, 123456.0])
    r = rounding.round_bf16(x)
    assert np.array_equal(rounding.round_bf16(r), r)
    assert np.all(np.abs(r - x) <= np.abs(x) * 2.0 ** -8)


def test_round_f32():
    assert rounding.round_f32(np.array([1.0 + 2.0 ** -30]))[0] == 1.0
    assert rounding.round_f32(np.array([0.1]))[0] == float(np.float32(0.1))


# ---------------------------------------------------------------- rmsnorm / silu
def test_rmsnorm_hand_value_and_library():
    x = np.array([[3.0, 4.0]])
    g = np.array([2.0, 0.5])
    got = model.rmsnorm(x, g, 0.0)
    s = math.sqrt(12.5)
    assert np.allclose(got, [[3.0 / s * 2.0, 4.0 / s * 0.5]], rtol=1e-15)
    rng = np.random.default_rng(1)
    x = rng.standard_normal((5, 64))
    g = rng.standard_normal(64)
    want = torch.nn.functional.rms_norm(torch.from_numpy(x), (64,), torch.from_numpy(g), 1e-5).numpy()
    assert np.allclose(model.rmsnorm(x, g, 1e-5), want, rtol=1e-13, atol=1e-15)


def test_silu_library_and_values():
    x = np.linspace(-8, 8, 101)
    assert np.allclose(model.silu(x), torch.nn.functional.silu(torch.from_numpy(x)).numpy(), rtol=1e-13)
    assert model.silu(np.array([0.0]))[0] == 0.0
    assert abs(model.silu(np.array([1.0]))[0] - 1.0 / (1.0 + math.exp(-1.0))) < 1e-16


# ---------------------------------------------------------------- rope
def test_rope_two_dim_is_a_plane_rotation():
    x = np.array([[[1.0, 0.0]]])           # [R=1, H=1, d_h=2]
    y = model.rope(x, np.array([3]), 10000.0)
    assert np.allclose(y[0, 0], [math.cos(3.0), math.sin(3.0)], atol=1e-15)


def test_rope_complex_form_norm_and_relative_position():
    rng = np.random.default_rng(2)
    dh, H, R = 16, 3, 7
    x = rng.standard_normal((R, H, dh))
    pos = rng.integers(0, 500, size=R)
    theta = 10000.0
    y = model.rope(x, pos, theta)
    # independent formulation: (x_j + i x_{j+dh/2}) * exp(i pos theta^(-2j/dh))
    half = dh // 2
    for r, h, j in itertools.product(range(R), range(H), range(half)):
        zc = complex(x[r, h, j], x[r, h, j + half]) * np.exp(1j * pos[r] * theta ** (-2.0 * j / dh))
        assert abs(y[r, h, j] - zc.real) < 1e-12 and abs(y[r, h, j + half] - zc.imag) < 1e-12
    assert np.allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-13)
    assert np.array_equal(model.rope(x, np.zeros(R, dtype=int), theta), x)
    # <rope(q, m), rope(k, n)> depends on m - n only
    q = rng.standard_normal((1, 1, dh))
    k = rng.standard_normal((1, 1, dh))
    d1 = np.sum(model.rope(q, [11], theta) * model.rope(k, [4], theta))
    d2 = np.sum(model.rope(q, [107], theta) * model.rope(k, [100], theta))
    assert abs(d1 - d2) < 1e-12


# ---------------------------------------------------------------- attention
def _attention_brute(q, K, V):
    M, H, dh = q.shape
    N = K.shape[0]
    out = np.zeros((M, H, dh))
    for m in range(M):
        for h in range(H):
            s = [sum(q[m, h, d] * K[n, h, d] for d in range(dh)) / math.sqrt(dh) for n in range(N)]
            mx = max(s)
            e = [math.exp(v - mx) for v in s]
            tot = sum(e)
            for d in range(dh):
                out[m, h, d] = sum(e[n] / tot * V[n, h, d] for n in range(N))
    return out


def test_attention_brute_force_tiny():
    rng = np.random.default_rng(3)
    q = rng.standard_normal((3, 2, 4))
    K = rng.standard_normal((8, 2, 4))
    V = rng.standard_normal((8, 2, 4))
    assert np.allclose(model.attention_rows(q, K, V), _attention_brute(q, K, V), rtol=1e-12, atol=1e-14)


def test_attention_library_row_subset_and_permutation():
    rng = np.random.default_rng(4)
    N, H, dh = 37, 3, 16
    Q = rng.standard_normal((N, H, dh))
    K = rng.standard_normal((N, H, dh))
    V = rng.standard_normal((N, H, dh))
    t = lambda a: torch.from_numpy(a).permute(1, 0, 2)[None]
    want = torch.nn.functional.scaled_dot_product_attention(t(Q), t(K), t(V))[0].permute(1, 0, 2).numpy()
    full = model.attention_rows(Q, K, V)
    assert np.allclose(full, want, rtol=1e-12, atol=1e-14)
    rows = np.array([30, 2, 17, 5])
    sub = model.attention_rows(Q[rows], K, V)
    assert np.allclose(sub, full[rows], rtol=1e-13, atol=1e-15)       # rows are independent
    perm = rng.permutation(N)                                          # key order is irrelevant
    assert np.allclose(model.attention_rows(Q[rows], K[perm], V[perm]), sub, rtol=1e-12, atol=1e-14)
    # a zero query attends uniformly: output = mean of V
    z = model.attention_rows(np.zeros((1, H, dh)), K, V)
    assert np.allclose(z[0], V.mean(axis=0), rtol=1e-13)


# ---------------------------------------------------------------- posterior
def test_log_softmax_library():
    rng = np.random.default_rng(5)
    z = rng.standard_normal((4, 1024)) * 3
    assert np.allclose(posterior.log_softmax(z), scipy.special.log_softmax(z, axis=-1), rtol=1e-13, atol=1e-13)
    assert np.allclose(np.exp(posterior.log_softmax(z)).sum(-1), 1.0, rtol=1e-13)
    # shift invariance and no overflow
    assert np.allclose(posterior.log_softmax(z + 1000.0), posterior.log_softmax(z), atol=1e-10)


def test_kl_closed_forms():
    a, b = 0.3, 0.6
    lp = np.log(np.array([[a, 1 - a]]))
    lq = np.log(np.array([[b, 1 - b]]))
    want = a * math.log(a / b) + (1 - a) * math.log((1 - a) / (1 - b))
    assert abs(posterior.kl_rows(lp, lq)[0] - want) < 1e-15
    # direction matters: KL(p||q) != KL(q||p)
    rev = b * math.log(b / a) + (1 - b) * math.log((1 - b) / (1 - a))
    assert abs(posterior.kl_rows(lq, lp)[0] - rev) < 1e-15 and abs(want - rev) > 1e-3
    # three-way against a uniform: KL(p||U) = log 3 - H(p)
    p = np.array([[0.5, 0.25, 0.25]])
    ent = -(p * np.log(p)).sum()
    assert abs(posterior.kl_rows(np.log(p), np.log(np.full((1, 3), 1 / 3)))[0] - (math.log(3) - ent)) < 1e-15
    # shifting every logit of a row by a constant changes nothing
    z = np.array([[0.2, -1.0, 3.0]]); z2 = np.array([[0.0, 0.5, 2.0]])
    k1 = posterior.kl_rows(posterior.log_softmax(z), posterior.log_softmax(z2))
    k2 = posterior.kl_rows(posterior.log_softmax(z + 7), posterior.log_softmax(z2 - 3))
    assert abs(k1[0] - k2[0]) < 1e-14


@pytest.mark.parametrize("V", [1024, 126464])
def test_kl_identities_and_library(V):
    rng = np.random.default_rng(V)
    z1 = rng.standard_normal((3, V)) * 2.0
    z0 = z1 + 0.3 * rng.standard_normal((3, V))
    lp, lq = posterior.log_softmax(z1), posterior.log_softmax(z0)
    D = posterior.kl_rows(lp, lq)
    assert np.all(D >= 0)
    assert np.all(posterior.kl_rows(lp, lp) == 0.0)
    # Pinsker: ||p - q||_1 <= sqrt(2 KL)   (appendix deriving A3)
    l1 = np.abs(np.exp(lp) - np.exp(lq)).sum(-1)
    assert np.all(l1 <= np.sqrt(2 * D) + 1e-12)
    want = scipy.special.rel_entr(np.exp(lp), np.exp(lq)).sum(-1)
    assert np.allclose(D, want, rtol=1e-10)
    tk = torch.nn.functional.kl_div(torch.from_numpy(lq), torch.from_numpy(lp), reduction="none",
                                    log_target=True).sum(-1).numpy()
    assert np.allclose(D, tk, rtol=1e-10)


def test_uncertainty_maxprob_argmax():
    z = np.array([[0.0, 2.0, 2.0, -1.0], [5.0, 1.0, 0.0, 5.0]])
    lp = posterior.log_softmax(z)
    e = np.exp(z[0]); p0 = e / e.sum()
    assert abs(posterior.max_prob(lp)[0] - p0.max()) < 1e-15
    assert abs(posterior.uncertainty(lp)[0] - (1 - p0.max())) < 1e-15
    assert list(posterior.argmax_lowest(z)) == [1, 0]          # ties -> lowest id
