"""Pins of the oracle's selection surrogate (Exp-5, the combined setting: a fixed fraction k of the
positions not yet locked is computed per step): the choice on a hand table and against brute
force, k = 1 == plain SureLock, and the invariants of a run (budget, masked slots of the block
always computed, skipped rows keep cache / posterior / score, KL against the last computed
posterior)."""
import math

import numpy as np
import pytest

from oracle import control, posterior, sampler
from oracle.model import Config
from paper_2602_06412_amd import workloads as wl


def _cfg(shape):
    return Config(shape.n_layers, shape.d_model, shape.n_heads, shape.d_head, shape.d_ff,
                  shape.vocab, shape.mask_id, shape.rms_eps, shape.rope_theta, shape.storage)


@pytest.fixture(scope="module")
def tiny():
    shape = wl.Shape("tiny", 2, 64, 2, 32, 176, 128, "fp32")
    w = wl.weights_to_numpy64(wl.make_weights(shape, seed=11, std=0.2, norm_gain_jitter=0.1))
    return _cfg(shape), w


def test_select_rows_by_hand_and_brute_force():
    masked = np.zeros(12, dtype=np.uint8); masked[[6, 7, 10]] = 1
    d_last = np.array([0.5, 0.1, np.inf, 0.3, 0.3, 0.0, 9, 9, 0.2, 0.7, 0, 0], dtype=np.float32)
    A = [0, 1, 2, 3, 4, 6, 7, 8, 9, 10]                       # 5 and 11 are locked
    # n = 10, k = 0.5 -> 5 rows: the two masked slots of block [6, 10) first, then by d_last: 2 (inf), 9, 0
    assert control.select_rows(A, masked, d_last, 6, 10, 0.5) == [0, 2, 6, 7, 9]
    # ties (3 and 4 at 0.3) go to the lower position; position 10 is masked but outside the block
    assert control.select_rows(A, masked, d_last, 6, 10, 0.6) == [0, 2, 3, 6, 7, 9]
    # the must rows alone may exceed the budget
    assert control.select_rows(A, masked, d_last, 6, 11, 0.1) == [6, 7, 10]
    assert control.select_rows(A, masked, d_last, 6, 10, 1.0) == A
    assert control.select_rows([], masked, d_last, 6, 10, 0.8) == []
    rng = np.random.default_rng(1)
    for trial in range(300):
        N = int(rng.integers(1, 30))
        lock = rng.random(N) < 0.3
        msk = (rng.random(N) < 0.4) & ~lock
        d = (rng.integers(0, 5, N) / 4).astype(np.float32)
        d[rng.random(N) < 0.2] = np.inf
        lo = int(rng.integers(0, N)); hi = int(rng.integers(lo, N + 1))
        k = float(rng.choice([0.1, 0.5, 0.8, 1.0]))
        A = np.flatnonzero(~lock)
        got = control.select_rows(A, msk, d, lo, hi, k)
        n = len(A)
        must = [p for p in A if msk[p] and lo <= p < hi]
        assert set(must) <= set(got) <= set(A) and got == sorted(got)
        assert len(got) == max(len(must), min(n, math.ceil(k * n)))
        others = [p for p in got if p not in must]
        left = [p for p in A if p not in got]
        for p in others:                                        # no skipped row outranks a chosen one
            for q in left:
                assert (d[p], -p) > (d[q], -q)


def _run_sel(cfg, w, eps, k, T=16, n_p=8, n_gen=16, seed=5):
    st = sampler.init_state(cfg, w, wl.prompt_uniform(seed, n_p, cfg.vocab, cfg.mask_id), n_gen)
    sched = sampler.block_schedule(n_p, n_gen, n_gen, T)
    recs, snaps = [], []
    for (lo, hi, kk) in sched:
        pre = (st.lock.copy(), st.masked.copy(), [a.copy() for a in st.Kc], st.prev_lp.copy(), st.d_last.copy())
        recs.append(sampler.surelock_step(cfg, w, st, eps, lo, hi, kk, select_k=k))
        snaps.append(pre)
    return st, recs, snaps


def test_selection_k_one_is_plain_surelock_and_run_invariants(tiny):
    cfg, w = tiny
    st0, recs0, _ = _run_sel(cfg, w, 2e-3, None)
    st1, recs1, _ = _run_sel(cfg, w, 2e-3, 1.0)
    assert np.array_equal(st0.lock, st1.lock) and np.array_equal(st0.tokens, st1.tokens)
    assert all(np.array_equal(a.logits, b.logits) for a, b in zip(recs0, recs1))
    st, recs, snaps = _run_sel(cfg, w, 2e-3, 0.8)
    assert st.masked.sum() == 0, "decoding must still finish: masked slots of the block are always computed"
    skipped_any = False
    for r, (lock, masked, Kc, plp, d_last) in zip(recs, snaps):
        A = np.flatnonzero(lock == 0)
        if r.t == 1:
            assert np.array_equal(r.active_pos, A)              # selection starts once scores exist
            continue
        n = len(A)
        must = [p for p in A if masked[p]]
        assert len(r.active_pos) == max(len(must), min(n, math.ceil(0.8 * n)))
        assert set(must) <= set(r.active_pos) <= set(A)
        assert set(r.F) <= set(r.active_pos)                    # only computed rows can lock
        skipped = np.setdiff1d(A, r.active_pos)
        skipped_any |= len(skipped) > 0
        j = recs.index(r)
        if j + 1 < len(snaps):
            nxt = snaps[j + 1]
            for p in skipped:                                   # a skipped row keeps cache, posterior, score
                assert np.array_equal(nxt[2][0][p], Kc[0][p]) and np.array_equal(nxt[3][p], plp[p])
                assert nxt[4][p] == d_last[p] and nxt[0][p] == 0
        # KL of a computed row is against the posterior it had when last computed
        lp = posterior.log_softmax(r.logits)
        assert np.allclose(r.kl, posterior.kl_rows(lp, plp[r.active_pos]), rtol=1e-12, atol=1e-15)
    assert skipped_any
    assert sum(len(r.active_pos) for r in recs) < sum(len(r.active_pos) for r in recs0)
