"""Pins of the oracle's temperature sampling: the Philox4x32-10 block function against the
known-answer vectors published with the generator (Random123 distribution of Salmon et al.,
SC'11, file kat_vectors), the uniform map, the Gumbel-max draw against softmax(z / tau) by a
chi-square test, the tau -> 0 limit, and what the paper's appendix on temperature states: the
lock decisions do not depend on tau."""
import numpy as np
import pytest

from oracle import posterior, sampler, sampling
from oracle.model import Config
from paper_2602_06412_amd import workloads as wl


def test_philox_known_answers():
    kat = [([0, 0, 0, 0], [0, 0], "6627e8d5 e169c58d bc57ac4c 9b00dbd8"),
           ([0xffffffff] * 4, [0xffffffff] * 2, "408f276d 41c83b0e a20bc7c6 6d5451fd"),
           ([0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344], [0xa4093822, 0x299f31d0],
            "d16cfe09 94fdcceb 5001e420 24126ea1")]
    for ctr, key, want in kat:
        assert " ".join(f"{x:08x}" for x in sampling.philox4x32_10(ctr, key)) == want
    # the vectorised form is the same function
    rng = np.random.default_rng(0)
    c = rng.integers(0, 2 ** 32, (4, 50), dtype=np.uint64)
    got = sampling.philox4x32_10_vec(c[0], c[1], c[2], c[3], 0x12345678, 0x9abcdef0)
    for i in range(50):
        assert [int(g[i]) for g in got] == sampling.philox4x32_10([int(c[j, i]) for j in range(4)], [0x12345678, 0x9abcdef0])


def test_uniforms_are_fp32_exact_open_interval_and_keyed():
    u = sampling.uniforms(seed=7, t=3, g=11, vocab=1001)
    assert u.shape == (1001,) and np.all(u > 0) and np.all(u < 1)
    assert np.array_equal(u, u.astype(np.float32).astype(np.float64))          # exact in fp32
    assert np.all((u * 2 ** 24) % 2 == 1)                                      # odd multiples of 2^-24
    assert abs(u.mean() - 0.5) < 0.03 and abs(u.var() - 1 / 12) < 0.01
    for other in (dict(seed=8), dict(t=4), dict(g=12)):
        kw = dict(seed=7, t=3, g=11, vocab=1001); kw.update(other)
        assert not np.array_equal(u, sampling.uniforms(**kw))
    assert np.array_equal(u[:500], sampling.uniforms(7, 3, 11, 500))           # word v does not depend on vocab


def test_gumbel_max_draw_follows_softmax_of_z_over_tau():
    z = np.array([2.0, 1.0, 0.5, 0.0, -1.0, 1.5, -3.0, 0.7])
    for tau in (0.5, 1.0, 2.0):
        p = np.exp(z / tau - np.max(z / tau)); p /= p.sum()
        n = 6000
        counts = np.bincount([sampling.sample_token(z, tau, seed=1, t=1, g=g) for g in range(n)], minlength=len(z))
        chi2 = float(np.sum((counts - n * p) ** 2 / (n * p)))
        assert chi2 < 29.9, (tau, chi2)            # 7 degrees of freedom: P(chi2 > 29.9) = 1e-4
    # tau -> 0: the draw is the argmax
    assert all(sampling.sample_token(z, 1e-6, 1, 1, g) == 0 for g in range(50))


def _cfg(shape):
    return Config(shape.n_layers, shape.d_model, shape.n_heads, shape.d_head, shape.d_ff,
                  shape.vocab, shape.mask_id, shape.rms_eps, shape.rope_theta, shape.storage)


def test_temperature_changes_tokens_not_the_first_lock_decisions():
    shape = wl.Shape("tiny", 2, 64, 2, 32, 176, 128, "fp32")
    w = wl.weights_to_numpy64(wl.make_weights(shape, seed=11, std=0.2, norm_gain_jitter=0.1))
    cfg = _cfg(shape)

    def run(tau):
        st = sampler.init_state(cfg, w, wl.prompt_uniform(5, 8, cfg.vocab, cfg.mask_id), 16)
        recs = [sampler.surelock_step(cfg, w, st, 2e-3, lo, hi, k, temperature=tau, seed=3)
                for (lo, hi, k) in sampler.block_schedule(8, 16, 16, 8)]
        return st, recs
    st0, r0 = run(0.0)
    st1, r1 = run(1.5)
    # step 1 sees the same state: identical posteriors, scores, chosen positions; only the written ids differ
    assert np.array_equal(r0[0].logits, r1[0].logits) and r0[0].unmasked == r1[0].unmasked and r0[0].F == r1[0].F
    assert np.array_equal(r0[0].write_id, r0[0].argmax)
    elig = [j for j, p in enumerate(r1[0].active_pos) if p >= 8]
    assert any(r1[0].write_id[j] != r1[0].argmax[j] for j in elig), "tau = 1.5 should move some draws off the argmax"
    assert all(r1[0].write_id[j] == r1[0].argmax[j] for j in range(len(r1[0].active_pos)) if j not in elig)
    for p in r1[0].unmasked:
        j = list(r1[0].active_pos).index(p)
        assert st1.tokens[p] != cfg.mask_id and (r1[1].t == 2)
        assert r1[0].write_id[j] == sampling.sample_token(r1[0].logits[j], 1.5, 3, 1, p)
    assert st1.masked.sum() == 0 and not np.array_equal(st0.tokens, st1.tokens)
