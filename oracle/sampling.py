"""Categorical sampling at temperature tau > 0 for the oracle (test infrastructure).

App. 'Interaction between sampling temperature and SureLock': tau enters only the step
that materialises discrete tokens; the lock test keeps the raw (tau = 1) posterior.  The
reading taken: UpdateMASK still picks its k positions by the confidence max_v p (raw
posterior), and writes at each a token drawn from softmax(z / tau) instead of the argmax.

The draw is the Gumbel-max form, argmax_v (z_v + tau * G_v) with G_v = -ln(-ln U_v), which
samples softmax(z / tau) exactly and turns the draw into an argmax that a GPU kernel can
take in one streaming pass.  U_v comes from the counter-based generator Philox4x32-10
(Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3", SC'11), which
both sides implement from its published definition: integer arithmetic only, so the
uniforms are bit-identical; the logarithms are taken in fp64 here.
"""
import numpy as np

_M0, _M1 = 0xD2511F53, 0xCD9E8D57
_W0, _W1 = 0x9E3779B9, 0xBB67AE85
_MASK = 0xFFFFFFFF


def philox4x32_10(counter, key):
    """One block of Philox4x32 with 10 rounds.  counter: 4 uint32, key: 2 uint32 -> 4 uint32."""
    c = [int(x) & _MASK for x in counter]
    k = [int(x) & _MASK for x in key]
    for _ in range(10):
        p0, p1 = _M0 * c[0], _M1 * c[2]
        hi0, lo0, hi1, lo1 = p0 >> 32, p0 & _MASK, p1 >> 32, p1 & _MASK
        c = [hi1 ^ c[1] ^ k[0], lo1, hi0 ^ c[3] ^ k[1], lo0]
        k = [(k[0] + _W0) & _MASK, (k[1] + _W1) & _MASK]
    return c


def philox4x32_10_vec(c0, c1, c2, c3, k0, k1):
    """The same block function on NumPy uint64 arrays (values < 2^32); returns four arrays."""
    c0, c1, c2, c3 = (np.asarray(x, dtype=np.uint64) for x in (c0, c1, c2, c3))
    k0, k1 = np.uint64(k0), np.uint64(k1)
    m = np.uint64(_MASK)
    for _ in range(10):
        p0, p1 = np.uint64(_M0) * c0, np.uint64(_M1) * c2          # < 2^64: no overflow
        hi0, lo0, hi1, lo1 = p0 >> np.uint64(32), p0 & m, p1 >> np.uint64(32), p1 & m
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
        k0, k1 = (k0 + np.uint64(_W0)) & m, (k1 + np.uint64(_W1)) & m
    return c0, c1, c2, c3


def uniforms(seed, t, g, vocab):
    """U_v in (0, 1) for v < vocab at step t and flat row id g: word v % 4 of the block with counter
    (v // 4, g, t, 0) and key (seed low word, seed high word); U = (2 (x >> 9) + 1) / 2^24, an odd
    multiple of 2^-24 (exact in fp32, never 0 or 1)."""
    nb = (vocab + 3) // 4
    blk = np.arange(nb, dtype=np.uint64)
    w = philox4x32_10_vec(blk, np.full(nb, g, np.uint64), np.full(nb, t, np.uint64), np.zeros(nb, np.uint64),
                          int(seed) & _MASK, (int(seed) >> 32) & _MASK)
    x = np.stack(w, axis=1).reshape(-1)[:vocab]
    return ((x >> np.uint64(9)) * np.uint64(2) + np.uint64(1)).astype(np.float64) * 2.0 ** -24


def perturbed_logits(z_row, tau, seed, t, g):
    """z_v + tau * G_v (fp64) for one row."""
    u = uniforms(seed, t, g, len(z_row))
    return np.asarray(z_row, dtype=np.float64) + tau * (-np.log(-np.log(u)))


def sample_token(z_row, tau, seed, t, g):
    """The token drawn for flat row g at step t: argmax of the perturbed logits, lowest id on ties."""
    return int(np.argmax(perturbed_logits(z_row, tau, seed, t, g)))
