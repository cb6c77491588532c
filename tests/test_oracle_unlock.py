"""Pins of the oracle's optional unlocking (App. 'Optional Unlocking'): the unlock rule on
hand-made tables (each conjunct alone, the strict inequalities, the percentile over the
active rows), the cool-down and the stricter re-lock threshold, the read-only probe against
the plain full forward, and what the appendix states about a run: an unlock leaves the
current step unchanged and the slot is recomputed from the next step on."""
import math

import numpy as np
import pytest

from oracle import control, model, posterior, sampler
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


# ---- the unlock rule, by hand ---------------------------------------------------------------
def test_unlock_rule_each_conjunct_and_strictness():
    # active uncertainties 0.1 .. 0.5: the 40th percentile by nearest rank is the 2nd smallest
    u_act = np.array([0.5, 0.1, 0.3, 0.2, 0.4], dtype=np.float32)
    theta = np.float32(0.2)
    lock_step = np.zeros(12, dtype=np.int64)
    pos = np.array([2, 3, 5, 7, 8, 9, 11])
    lock_step[pos] = [4, 4, 4, 4, 4, 7, 6]
    #                 ok    u==th  u<th  D==eps D<eps  young  t-t*==Dint
    u_p = np.array([0.30, theta, 0.10, 0.30, 0.30, 0.90, 0.90], dtype=np.float32)
    D_p = np.array([0.50, 0.50, 0.50, 0.25, 0.10, 0.90, 0.90], dtype=np.float32)
    got = control.unlock_rule(lock_step, pos, u_p, D_p, u_act, 40.0, np.float32(0.25), t=10, d_interval=4)
    assert got == [2]
    # one step later the slot locked at t* = 6 has t - t* = 5 > 4
    got = control.unlock_rule(lock_step, pos, u_p, D_p, u_act, 40.0, np.float32(0.25), t=11, d_interval=4)
    assert got == [2, 11]
    # m = 100 puts theta at the largest active u: only probes above every active row pass
    got = control.unlock_rule(lock_step, pos, u_p, D_p, u_act, 100.0, np.float32(0.25), t=20, d_interval=4)
    assert got == [9, 11]
    # no active row: theta = -inf, the first conjunct is vacuous
    got = control.unlock_rule(lock_step, pos, u_p, D_p, np.zeros(0, np.float32), 40.0, np.float32(0.25), 20, 4)
    assert got == [2, 3, 5, 9, 11]
    # eps_unlock = +inf: nothing can unlock
    assert control.unlock_rule(lock_step, pos, u_p, D_p, u_act, 40.0, np.float32(np.inf), 20, 0) == []


def test_unlock_rule_against_brute_force():
    rng = np.random.default_rng(3)
    for trial in range(200):
        n_act, n_p = int(rng.integers(0, 9)), int(rng.integers(0, 9))
        u_act = rng.integers(0, 6, n_act).astype(np.float32) / 8
        N = 20
        pos = np.sort(rng.choice(N, n_p, replace=False))
        lock_step = rng.integers(1, 8, N)
        u_p = rng.integers(0, 6, n_p).astype(np.float32) / 8
        D_p = rng.integers(0, 4, n_p).astype(np.float32) / 4
        m = float(rng.choice([1, 20, 50, 99, 100]))
        t, d_int, eps_u = int(rng.integers(5, 12)), int(rng.integers(0, 5)), np.float32(rng.integers(0, 4) / 4)
        if n_act:
            srt = np.sort(u_act)
            theta = srt[max(1, math.ceil(m * n_act / 100)) - 1]
        else:
            theta = -np.inf
        want = [int(p) for j, p in enumerate(pos) if u_p[j] > theta and D_p[j] > eps_u and t - lock_step[p] > d_int]
        assert control.unlock_rule(lock_step, pos, u_p, D_p, u_act, m, eps_u, t, d_int) == want


# ---- re-locking: cool-down and the stricter threshold ---------------------------------------
def test_lock_rule_cooldown_and_rho():
    lock = np.zeros(6, dtype=np.uint8)
    masked = np.zeros(6, dtype=np.uint8)
    pos = np.arange(6)
    eps, rho = np.float32(0.1), 0.5
    relocked = np.array([0, 1, 1, 1, 1, 0], dtype=np.uint8)
    cool = np.array([0, 0, 0, 7, 8, 0])
    #              plain   <=rho*eps  between   cooled(t>7)  cooling(t<=8)  > eps
    D = np.array([0.10, 0.05, 0.07, 0.01, 0.01, 0.2], dtype=np.float32)
    u = np.zeros(6, dtype=np.float32)
    F = control.lock_rule(lock, masked, pos, D, u, eps, first_step=False, relocked=relocked, cool_until=cool,
                          rho=rho, t=8)
    assert F == [0, 1, 3]
    # without the unlocking state the same call is the plain rule
    assert control.lock_rule(lock, masked, pos, D, u, eps, first_step=False) == [0, 1, 2, 3, 4]
    # rho = 1 and an expired cool-down give the plain rule back
    F = control.lock_rule(lock, masked, pos, D, u, eps, first_step=False, relocked=relocked, cool_until=cool,
                          rho=1.0, t=9)
    assert F == [0, 1, 2, 3, 4]


# ---- the probe --------------------------------------------------------------------------------
def test_probe_forward_reads_cache_and_writes_nothing(tiny):
    cfg, w = tiny
    N = 24
    tokens = np.concatenate([wl.prompt_uniform(3, 8, cfg.vocab, cfg.mask_id), np.full(16, cfg.mask_id)])
    z_full, Ks, Vs = model.forward_full(cfg, w, tokens)
    Kc, Vc = [k.copy() for k in Ks], [v.copy() for v in Vs]
    rows = np.array([0, 5, 6, 17, 23])
    z = model.forward_active(cfg, w, tokens, rows, Kc, Vc, write_cache=False)
    # with the cache holding the K/V of these very tokens the probe is the full forward on those rows
    assert np.allclose(z, z_full[rows], rtol=0, atol=2e-6)
    for l in range(cfg.n_layers):
        assert np.array_equal(Kc[l], Ks[l]) and np.array_equal(Vc[l], Vs[l])
    # rows are independent of which other rows are probed with them
    z1 = model.forward_active(cfg, w, tokens, rows[2:3], Kc, Vc, write_cache=False)
    assert np.array_equal(z1[0], z[2])
    # a stale own key/value shows in the probe (the row attends to the cached entry, not a fresh one)
    Kc[0][6] += 0.5
    z2 = model.forward_active(cfg, w, tokens, rows, Kc, Vc, write_cache=False)
    assert not np.allclose(z2[2], z[2])


# ---- runs ---------------------------------------------------------------------------------------
def _run(cfg, w, eps, unlock, T=16, n_p=8, n_gen=16, seed=5):
    st = sampler.init_state(cfg, w, wl.prompt_uniform(seed, n_p, cfg.vocab, cfg.mask_id), n_gen)
    sched = sampler.block_schedule(n_p, n_gen, n_gen, T)
    recs, snaps = [], []
    for (lo, hi, kk) in sched:
        pre = (st.lock.copy(), [a.copy() for a in st.Kc], [a.copy() for a in st.Vc], st.prev_lp.copy())
        rec = sampler.surelock_step(cfg, w, st, eps, lo, hi, kk, unlock=unlock)
        recs.append(rec)
        snaps.append((pre, st.lock.copy(), st.tokens.copy(), [a.copy() for a in st.Kc], [a.copy() for a in st.Vc],
                      st.prev_lp.copy(), st.relocked.copy(), st.cool_until.copy(), st.lock_step.copy()))
    return st, recs, snaps


def test_unlocking_that_never_fires_is_plain_surelock(tiny):
    cfg, w = tiny
    never = sampler.UnlockParams(period=1, m=50.0, eps_unlock=np.inf, d_interval=0, d_cool=0, rho=1.0)
    st0, recs0, _ = _run(cfg, w, 2e-3, None)
    st1, recs1, _ = _run(cfg, w, 2e-3, never)
    assert st0.lock.sum() > 0
    assert np.array_equal(st0.lock, st1.lock) and np.array_equal(st0.tokens, st1.tokens)
    for a, b in zip(recs0, recs1):
        assert np.array_equal(a.logits, b.logits) and a.F == b.F
        assert b.probe is not None and b.probe.unlocked == []
        assert np.all(b.probe.D >= -1e-12)


def test_unlocking_run_invariants(tiny):
    cfg, w = tiny
    # an eager rule (every probed slot past the interval whose uncertainty tops the least
    # uncertain active row unlocks) so that unlock events do occur on this tiny model
    prm = sampler.UnlockParams(period=2, m=1.0, eps_unlock=0.0, d_interval=1, d_cool=2, rho=0.5)
    st, recs, snaps = _run(cfg, w, 5e-3, prm, T=16)
    events = [(r.t, p) for r in recs if r.probe for p in r.probe.unlocked]
    assert events, "workload must exercise unlocking"
    assert all(r.probe is None for r in recs if r.t % 2) and all(r.probe is not None for r in recs if r.t % 2 == 0)
    relocks = 0
    for r, snap in zip(recs, snaps):
        pre, lock_after, tokens, Kc, Vc, plp, relocked, cool, lock_step = snap
        lock_before = pre[0]
        assert np.array_equal(r.active_pos, np.flatnonzero(lock_before == 0))
        if r.probe is None:
            assert np.all(lock_after >= lock_before)
            continue
        pr = r.probe
        locked_now = lock_before.copy(); locked_now[r.F] = 1
        assert np.array_equal(pr.pos, np.flatnonzero(locked_now))            # every locked row is probed
        for p in pr.unlocked:
            assert lock_after[p] == 0 and relocked[p] == 1 and cool[p] == r.t + prm.d_cool
            assert r.t - lock_step[p] > prm.d_interval
        # the probe left this step as it was: the cache and the kept posteriors of probed rows are unchanged
        # by it (they equal what the step's own forward left, which touches only active rows)
        for p in pr.pos:
            if p not in r.active_pos:
                for l in range(cfg.n_layers):
                    assert np.array_equal(Kc[l][p], pre[1][l][p]) and np.array_equal(Vc[l][p], pre[2][l][p])
                assert np.array_equal(plp[p], pre[3][p])
        # D~ is the KL against the posterior kept from the lock step
        lp = posterior.log_softmax(pr.logits)
        assert np.allclose(pr.D, posterior.kl_rows(lp, plp[pr.pos]), rtol=1e-12, atol=1e-15)
    for (t_u, p) in events:
        nxt = recs[t_u]                                                      # step t_u + 1
        assert p in nxt.active_pos                                            # recomputed from the next step on
        for r in recs[t_u:t_u + prm.d_cool]:
            assert p not in r.F                                               # cool-down
        later = [r for r in recs[t_u + prm.d_cool:] if p in r.F]
        for r in later[:1]:
            j = list(r.active_pos).index(p)
            assert np.float32(r.kl[j]) <= np.float32(prm.rho) * np.float32(5e-3)   # stricter re-lock
            relocks += 1
    # K/V of an unlocked slot are rewritten at the next step (the invalidation)
    t_u, p = events[0]
    K_before = snaps[t_u - 1][3][0][p]
    K_after = snaps[t_u][3][0][p]
    tokens_changed = not np.array_equal(snaps[t_u - 1][2], snaps[max(t_u - 2, 0)][2])
    assert K_after.shape == K_before.shape and np.isfinite(K_after).all()
    assert tokens_changed or np.allclose(K_after, K_before)

