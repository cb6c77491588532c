"""GPU parity of optional unlocking (App. 'Optional Unlocking') against the oracle.

Kernel level, on synthetic fp32 inputs (bit-exact): the lock rule with cool-down / stricter
re-lock threshold / lock-time recording, and the unlock rule with its percentile over the active
rows, its three strict tests and the carry of the kept posterior row.
Run level, teacher-forced like the step tests: every step and every probe receives the oracle's
state; the probe's logits are compared within the logit tolerance, its scores in situ with the
fp64 formulas on the device's own logits, its decisions with the oracle's rule applied to the
device's own scores; the K/V cache and the posterior store must come out of the probe unchanged
(but for carried rows)."""
import numpy as np
import pytest
import torch

from oracle import control, posterior, sampler
from paper_2602_06412_amd import binding as B
from paper_2602_06412_amd import workloads as wl
from tests.gpu_util import DEV, check_logits, dev, oracle_cfg, weights_to_device
from tests.trajectory import run_oracle_unlock

pytestmark = pytest.mark.gpu


def _u32(conf):
    return np.maximum(np.float32(0), np.float32(1) - conf.astype(np.float32)).astype(np.float32)


# ---- kernel level ---------------------------------------------------------------------------------
@pytest.mark.parametrize("Bn,N,gate,t,ties", [(1, 128, 0.0, 5, False), (3, 333, 0.0, 9, True), (8, 1024, 20.0, 7, False),
                                              (2, 2048, 50.0, 4, True), (2, 64, 0.0, 1, False), (1, 15360, 7.0, 3, False)])
def test_lock_rule_relock(Bn, N, gate, t, ties):
    rng = np.random.default_rng(N * 13 + t)
    lock = (rng.random((Bn, N)) < 0.4).astype(np.uint8)
    masked = ((rng.random((Bn, N)) < 0.3) & (lock == 0)).astype(np.uint8)
    relocked = (rng.random((Bn, N)) < 0.5).astype(np.uint8)
    cool = rng.integers(0, 2 * t + 1, (Bn, N)).astype(np.int32)
    cool[0, :4] = [t - 1, t, t + 1, 0]                               # the boundary: lockable iff t > cool_until
    t_lock0 = rng.integers(0, t, (Bn, N)).astype(np.int32)
    idx, cu = control.compact_active(lock)
    M = len(idx)
    conf = rng.random(M).astype(np.float32)
    if ties:
        conf = (np.floor(conf * 8) / 8).astype(np.float32)
    kl = (rng.random(M) * 2e-3).astype(np.float32)
    eps = (rng.random(Bn) * 2e-3).astype(np.float32)
    rho = np.float32(0.6)
    kl[:min(M, 2)] = [rho * eps[idx[0] // N], eps[idx[0] // N]][:min(M, 2)]    # equality with either threshold
    u = _u32(conf)
    want, want_tl = lock.copy(), t_lock0.copy()
    for b in range(Bn):
        r0, r1 = cu[b], cu[b + 1]
        F = control.lock_rule(lock[b], masked[b], idx[r0:r1] - b * N, kl[r0:r1], u[r0:r1], eps[b], t == 1,
                              gate_m=float(np.float32(gate)) if gate > 0 else None, relocked=relocked[b],
                              cool_until=cool[b], rho=float(rho), t=t)
        want[b, F] = 1
        want_tl[b, F] = t
    for alias in (False, True):
        lock_d = dev(lock.reshape(-1))
        out = lock_d if alias else torch.full((Bn * N,), 7, dtype=torch.uint8, device=DEV)
        tl = dev(t_lock0.reshape(-1))
        B.sl_lock_rule_relock(lock_d, dev(masked.reshape(-1)), dev(idx, torch.int32), dev(cu, torch.int32), Bn * N,
                              dev(kl), dev(conf), dev(eps), gate, dev(relocked.reshape(-1)), dev(cool.reshape(-1)),
                              float(rho), t, Bn, N, out, tl)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy().reshape(Bn, N), want)
        assert np.array_equal(tl.cpu().numpy().reshape(Bn, N), want_tl)
    if t > 1:
        assert want.sum() > lock.sum(), "the case should lock something"
        # the re-lock state does change the outcome in these cases
        plain = lock.copy()
        for b in range(Bn):
            r0, r1 = cu[b], cu[b + 1]
            plain[b, control.lock_rule(lock[b], masked[b], idx[r0:r1] - b * N, kl[r0:r1], u[r0:r1], eps[b], False,
                                       gate_m=float(np.float32(gate)) if gate > 0 else None)] = 1
        assert not np.array_equal(plain, want)


def _session(shape, Bn, N, seed=1, **kw):
    w = wl.make_weights(shape, seed=seed, **kw)
    return w, B.Session(shape, weights_to_device(w), Bn, N).unlock_state()


@pytest.mark.parametrize("Bn,N,m,t,ties,p_lock", [(1, 128, 20.0, 10, False, 0.5), (3, 100, 50.0, 7, True, 0.3),
                                                  (2, 256, 60.0, 12, True, 0.6), (2, 64, 1.0, 9, False, 1.0),
                                                  (4, 96, 33.3, 8, True, 0.0)])
def test_unlock_rule_and_posterior_carry(Bn, N, m, t, ties, p_lock):
    shape = wl.C1
    _, sess = _session(shape, Bn, N)
    try:
        rng = np.random.default_rng(N * 17 + t)
        V, R = shape.vocab, Bn * N
        lock = (rng.random((Bn, N)) < p_lock).astype(np.uint8)
        t_lock = np.where(lock == 1, rng.integers(1, t + 1, (Bn, N)), 0).astype(np.int32)
        a_idx, a_cu = control.compact_active(lock)
        p_idx, p_cu = control.compact_active(1 - lock)
        Ma, Mp = len(a_idx), len(p_idx)
        conf_a = rng.random(Ma).astype(np.float32)
        conf_p = rng.random(Mp).astype(np.float32)
        kl_p = rng.random(Mp).astype(np.float32)
        if ties:
            conf_a = (np.floor(conf_a * 8) / 8).astype(np.float32)
            conf_p = (np.floor(conf_p * 8) / 8).astype(np.float32)
            kl_p = (np.floor(kl_p * 4) / 4).astype(np.float32)
        eps_u, d_int, d_cool = np.float32(0.25), 2, 3
        relocked0 = (rng.random((Bn, N)) < 0.2).astype(np.uint8)
        cool0 = rng.integers(0, 5, (Bn, N)).astype(np.int32)
        want_lock, want_rel, want_cool = lock.copy(), relocked0.copy(), cool0.copy()
        want_flag = np.zeros(Mp, dtype=np.uint8)
        for b in range(Bn):
            q0, q1 = p_cu[b], p_cu[b + 1]
            pos = p_idx[q0:q1] - b * N
            un = control.unlock_rule(t_lock[b], pos, _u32(conf_p[q0:q1]), kl_p[q0:q1],
                                     _u32(conf_a[a_cu[b]:a_cu[b + 1]]), float(np.float32(m)), eps_u, t, d_int)
            want_lock[b, un] = 0
            want_rel[b, un] = 1
            want_cool[b, un] = t + d_cool
            want_flag[q0:q1] = np.isin(pos, un)
        # a recognisable posterior store
        store = sess.post.view(sess.T)
        per = store.numel() // 2
        fill = torch.arange(2 * per, device=DEV, dtype=torch.float32).remainder(8191.0).to(sess.T)
        store.copy_(fill)
        before = store.clone()
        lock_d, rel_d, cool_d = dev(lock.reshape(-1)), dev(relocked0.reshape(-1)), dev(cool0.reshape(-1))
        flags = torch.full((R,), 9, dtype=torch.uint8, device=DEV)
        pad = lambda a, dt: dev(np.concatenate([a, np.zeros(R - len(a), a.dtype)]), dt)
        B.sl_unlock_rule(sess.ctx, lock_d, rel_d, cool_d, dev(t_lock.reshape(-1)), pad(p_idx, torch.int32),
                         dev(p_cu, torch.int32), R, pad(kl_p, None), pad(conf_p, None), dev(a_cu, torch.int32), R,
                         pad(conf_a, None), m, float(eps_u), t, d_int, d_cool, flags)
        torch.cuda.synchronize()
        assert np.array_equal(lock_d.cpu().numpy().reshape(Bn, N), want_lock)
        assert np.array_equal(rel_d.cpu().numpy().reshape(Bn, N), want_rel)
        assert np.array_equal(cool_d.cpu().numpy().reshape(Bn, N), want_cool)
        assert np.array_equal(flags[:Mp].cpu().numpy(), want_flag)
        if Mp and p_lock < 1.0:
            assert 0 < want_flag.sum() < Mp, "the case should unlock some rows and keep some"
        # carry: an unlocked row kept in the buffer step t + 1 will not read is copied across; nothing else moves
        want_store = before.clone().view(2, per)
        for r in np.flatnonzero(want_flag):
            g = int(p_idx[r])
            src, dst = int(t_lock.reshape(-1)[g]) & 1, t & 1
            if src != dst:
                want_store[dst, g * V:(g + 1) * V] = before.view(2, per)[src, g * V:(g + 1) * V]
        assert torch.equal(store.view(2, per), want_store)
    finally:
        sess.close()


def test_unlock_argument_errors():
    shape = wl.C1
    _, sess = _session(shape, 1, 128)
    try:
        z8 = torch.zeros(128, dtype=torch.uint8, device=DEV)
        zi = torch.zeros(129, dtype=torch.int32, device=DEV)
        zf = torch.zeros(128, device=DEV)
        for kw in (dict(percentile=0.0), dict(percentile=101.0), dict(t=0), dict(d_interval=-1), dict(d_cool=-1)):
            a = dict(percentile=20.0, t=3, d_interval=1, d_cool=1)
            a.update(kw)
            with pytest.raises(B.SureLockError):
                B.sl_unlock_rule(sess.ctx, z8, z8, zi, zi, zi, zi, 128, zf, zf, zi, 128, zf, a["percentile"], 0.1, a["t"],
                                 a["d_interval"], a["d_cool"], z8)
        for rho in (0.0, 1.5):
            with pytest.raises(B.SureLockError):
                B.sl_lock_rule_relock(z8, z8, zi, zi, 128, zf, zf, zf, 0.0, z8, zi, rho, 2, 1, 128, z8, zi)
        with pytest.raises(B.SureLockError):                                   # probe_logits missing
            B.sl_unlock_probe(sess.ctx, zi, z8, zi, 128, zi, zi, None, zf, zf, zi, sess.workspace)
        with pytest.raises(B.SureLockError):                                   # m_upper beyond B*N
            B.sl_unlock_probe(sess.ctx, zi, z8, zi, 129, zi, zi, sess.probe_logits, zf, zf, zi, sess.workspace)
    finally:
        sess.close()


# ---- run level ---------------------------------------------------------------------------------------
def _check_unlock_run(shape, w, steps, Bn, N, eps, prm, strict):
    V = shape.vocab
    sess = B.Session(shape, weights_to_device(w), Bn, N).unlock_state()
    n_events = n_probes = n_carried = 0
    try:
        eps_d = dev(np.asarray(eps, dtype=np.float32))
        last_logits = np.zeros((Bn * N, V))                      # the device's own newest logits per position
        undecided = set()                                        # rows whose unlock decision differed from the oracle's
        for us in steps:
            st = us.base
            lo, hi, k = st.block
            tokens = dev(st.tokens_in.reshape(-1), torch.int32)
            masked = dev(st.masked_in.reshape(-1).astype(np.uint8))
            lock = dev(st.lock_in.reshape(-1).astype(np.uint8))
            sess.t_lock.copy_(dev(us.t_lock_in.reshape(-1), torch.int32))
            sess.relocked.copy_(dev(us.relocked_in.reshape(-1).astype(np.uint8)))
            sess.cool_until.copy_(dev(us.cool_in.reshape(-1), torch.int32))
            sess.step_unlockable(tokens, masked, lock, eps_d, st.t, lo, hi, k, prm.rho)
            torch.cuda.synchronize()
            M = int(sess.cu_active[-1].item())
            idx = sess.active_idx[:M].cpu().numpy()
            assert np.array_equal(idx, st.active_idx), f"t={st.t}"
            z_gpu = sess.logits_view(st.t)[torch.as_tensor(idx, device=DEV, dtype=torch.long)].double().cpu().numpy()
            check_logits(z_gpu, st.logits, shape.storage, f"t={st.t}")
            kl = sess.kl[:M].cpu().numpy()
            conf = sess.conf[:M].cpu().numpy()
            am = sess.argmax[:M].cpu().numpy()
            if st.t > 1:
                # a row unlocked earlier is scored against the last posterior kept for it (p_{t*})
                want = posterior.kl_rows(posterior.log_softmax(z_gpu), posterior.log_softmax(last_logits[idx]))
                # (not checkable where the device, on its own scores, left a row locked that the oracle
                # unlocked: the next step is teacher-forced to treat it as unlocked, without the carry)
                ok = (np.abs(kl - want) <= 1e-4 * want + 2e-7) | np.isin(idx, sorted(undecided))
                undecided.clear()
                bad = np.flatnonzero(~ok)
                assert len(bad) == 0, (f"t={st.t}: rows {idx[bad][:8]} kl {kl[bad][:8]} want {want[bad][:8]} "
                                       f"t_lock {us.t_lock_in.reshape(-1)[idx[bad]][:8]} "
                                       f"relocked {us.relocked_in.reshape(-1)[idx[bad]][:8]}")
            last_logits[idx] = z_gpu
            # the rule that counts, on the device's own scores
            want_msk, want_tok = st.masked_in.copy().astype(np.uint8), st.tokens_in.copy()
            want_lock, want_tl = st.lock_in.copy(), us.t_lock_in.copy()
            for b in range(Bn):
                r0, r1 = st.cu_active[b], st.cu_active[b + 1]
                pos = st.active_idx[r0:r1] - b * N
                control.update_mask(want_msk[b], want_tok[b], pos, conf[r0:r1], am[r0:r1], lo, hi, k)
                F = control.lock_rule(st.lock_in[b], want_msk[b], pos, kl[r0:r1], _u32(conf[r0:r1]), np.float32(eps[b]),
                                      st.t == 1, relocked=us.relocked_in[b], cool_until=us.cool_in[b], rho=prm.rho,
                                      t=st.t)
                want_lock[b, F] = 1
                want_tl[b, F] = st.t
            assert np.array_equal(lock.cpu().numpy().reshape(Bn, N), want_lock), f"t={st.t}"
            assert np.array_equal(sess.t_lock.cpu().numpy().reshape(Bn, N), want_tl), f"t={st.t}"
            if st.t % prm.period:
                assert all(p is None for p in us.probe)
                continue
            # ---- the probe, on the oracle's state after the step ----
            n_probes += 1
            tokens = dev(st.tokens_out.reshape(-1), torch.int32)
            lock = dev(us.lock_mid.reshape(-1).astype(np.uint8))
            sess.t_lock.copy_(dev(us.t_lock_mid.reshape(-1), torch.int32))
            kv_before, post_before = sess.kv.clone(), sess.post.clone()
            sess.unlock_probe(tokens, lock, st.t, prm.m, prm.eps_unlock, prm.d_interval, prm.d_cool)
            torch.cuda.synchronize()
            p_idx = np.concatenate([p.pos + b * N for b, p in enumerate(us.probe)]).astype(np.int64)
            p_cu = np.concatenate([[0], np.cumsum([len(p.pos) for p in us.probe])])
            Mp = int(sess.cu_probe[-1].item())
            assert Mp == len(p_idx) and np.array_equal(sess.cu_probe.cpu().numpy(), p_cu)
            assert np.array_equal(sess.probe_idx[:Mp].cpu().numpy(), p_idx)
            assert torch.equal(sess.kv, kv_before), "the probe must not write the K/V cache"
            flags = sess.unlocked[:Mp].cpu().numpy()
            if Mp == 0:
                assert torch.equal(sess.post, post_before)
                continue
            zp = sess.probe_logits[:Mp].double().cpu().numpy()
            check_logits(zp, np.concatenate([p.logits for p in us.probe]), shape.storage, f"probe t={st.t}")
            lp = posterior.log_softmax(zp)
            kl_p, conf_p = sess.probe_kl[:Mp].cpu().numpy(), sess.probe_conf[:Mp].cpu().numpy()
            assert np.array_equal(sess.probe_argmax[:Mp].cpu().numpy(), posterior.argmax_lowest(zp))
            assert np.allclose(conf_p, posterior.max_prob(lp), rtol=2e-6)
            want = posterior.kl_rows(lp, posterior.log_softmax(last_logits[p_idx]))       # against p_{t*}
            assert np.all(np.abs(kl_p - want) <= 1e-4 * want + 2e-7), f"probe t={st.t}"
            # decisions: the oracle's rule on the device's own scores
            want_lock, want_rel, want_cool = us.lock_mid.copy(), us.relocked_in.copy(), us.cool_in.copy()
            want_flag = np.zeros(Mp, dtype=np.uint8)
            for b in range(Bn):
                q0, q1 = p_cu[b], p_cu[b + 1]
                pos = us.probe[b].pos
                un = control.unlock_rule(us.t_lock_mid[b], pos, _u32(conf_p[q0:q1]), kl_p[q0:q1],
                                         _u32(conf[st.cu_active[b]:st.cu_active[b + 1]]), prm.m,
                                         np.float32(prm.eps_unlock), st.t, prm.d_interval)
                want_lock[b, un] = 0
                want_rel[b, un] = 1
                want_cool[b, un] = st.t + prm.d_cool
                want_flag[q0:q1] = np.isin(pos, un)
                if strict:
                    # fp32 model: the device decides as the oracle did, rows on a threshold aside
                    o = us.probe[b]
                    theta = control.percentile_nearest_rank(
                        (1.0 - st.conf[st.cu_active[b]:st.cu_active[b + 1]]).astype(np.float32), prm.m)
                    near = (np.abs(o.D - prm.eps_unlock) <= 1e-6) | (np.abs(o.u - theta) <= 1e-6)
                    kept = set(int(p) for p in pos[~near])
                    assert set(int(p) for p in un if p in kept) == set(int(p) for p in o.unlocked if p in kept)
            assert np.array_equal(flags, want_flag), f"probe t={st.t}"
            oracle_flag = np.concatenate([np.isin(p.pos, p.unlocked) for p in us.probe])
            undecided.update(int(g) for g in p_idx[flags.astype(bool) != oracle_flag])
            assert len(undecided) <= max(2, Mp // 10), "decisions on the device's scores should rarely differ"
            assert np.array_equal(lock.cpu().numpy().reshape(Bn, N), want_lock)
            assert np.array_equal(sess.relocked.cpu().numpy().reshape(Bn, N), want_rel)
            assert np.array_equal(sess.cool_until.cpu().numpy().reshape(Bn, N), want_cool)
            n_events += int(want_flag.sum())
            # the posterior store: only carried rows change, and they now hold the kept row (compared as bytes:
            # rows no step has written yet hold whatever the allocator left, NaN patterns included)
            per = sess.post.numel() // 2
            rb = V * sess.post.view(sess.T).element_size()
            now, was = sess.post.view(2, per), post_before.view(2, per)
            want_store = was.clone()
            for r in np.flatnonzero(want_flag):
                g = int(p_idx[r])
                src, dst = int(us.t_lock_mid.reshape(-1)[g]) & 1, st.t & 1
                if src != dst:
                    want_store[dst, g * rb:(g + 1) * rb] = was[src, g * rb:(g + 1) * rb]
                    n_carried += 1
            if not torch.equal(now, want_store):
                diff = (now != want_store)[:, :Bn * N * rb].view(2, -1, rb).any(dim=2).nonzero().cpu().numpy()
                raise AssertionError(f"probe t={st.t}: posterior rows changed beyond the carried ones: (buffer, row) "
                                     f"{diff[:10].tolist()} of {len(diff)}; probed rows {p_idx[:10].tolist()}")
    finally:
        sess.close()
    return n_probes, n_events, n_carried


def test_c1_fp32_run_with_unlocking():
    """Config-1 geometry on the shape-generic kernels, weights scaled up (std 0.2) so that posteriors
    are peaked and the KL rule, the probe and the unlock rule all fire on their own."""
    shape = wl.C1
    w = wl.make_weights(shape, seed=1, std=0.2, norm_gain_jitter=0.05)
    cfg, w64 = oracle_cfg(shape), wl.weights_to_numpy64(w)
    prm = sampler.UnlockParams(period=3, m=50.0, eps_unlock=5e-4, d_interval=1, d_cool=2, rho=0.7)
    eps = [1e-3]
    steps = run_oracle_unlock(cfg, w64, [wl.prompt_uniform(7, 32, shape.vocab, shape.mask_id)], 96, 32, 96, eps, prm)
    assert sum(len(p.unlocked) for s in steps for p in s.probe if p) > 10
    relocks = sum(int((s.base.lock_rule_out.astype(bool) & ~s.base.lock_in.astype(bool) & s.relocked_in.astype(bool)).sum())
                  for s in steps)
    assert relocks > 0, "some unlocked position should lock again"
    n_probes, n_events, n_carried = _check_unlock_run(shape, w, steps, 1, 128, eps, prm, strict=True)
    assert n_probes == 10 and n_events > 10 and n_carried > 0


@pytest.mark.parametrize("Bn,n_p,n_gen,T,block,M_end", [(1, 72, 128, 16, 64, [24]), (3, 40, 96, 12, 96, [16, 50, 100])])
def test_bf16_run_with_unlocking_forced_schedule(Bn, n_p, n_gen, T, block, M_end):
    """The bf16 / MFMA route: a forced lock schedule supplies locked rows at every step (the KL rule is
    recorded and checked in situ), the probe and the unlock rule run every second step."""
    shape = wl.S_BF16
    w = wl.make_weights(shape, seed=3, norm_gain_jitter=0.05)
    cfg, w64 = oracle_cfg(shape), wl.weights_to_numpy64(w)
    prm = sampler.UnlockParams(period=2, m=30.0, eps_unlock=1e-3, d_interval=1, d_cool=2, rho=0.5)
    prompts = [wl.prompt_zipf(20 + b, n_p, shape.vocab, shape.mask_id) for b in range(Bn)]
    eps = [[1e-4, 1e-3, 1e-2][b % 3] for b in range(Bn)]
    steps = run_oracle_unlock(cfg, w64, prompts, n_gen, T, block, eps, prm, forced_M_end=M_end, seed=4)
    for s in steps:                                                   # the driver's bookkeeping
        un = np.zeros_like(s.lock_mid)
        for b, p in enumerate(s.probe):
            if p is not None:
                un[b, p.unlocked] = 1
        assert np.array_equal(s.lock_out, s.lock_mid & ~un.astype(bool))
    n_probes, n_events, n_carried = _check_unlock_run(shape, w, steps, Bn, n_p + n_gen, eps, prm, strict=False)
    assert n_probes == T // 2 and n_events > 0 and n_carried > 0


@pytest.mark.parametrize("gate", [0.0, 20.0])
def test_relock_rule_without_unlock_history_is_the_plain_rule(gate):
    """No position unlocked before, no cool-down running, rho = 1: sl_lock_rule_relock must give what
    sl_lock_rule / sl_lock_rule_gated give on the same inputs (and record the lock step)."""
    Bn, N, t = 3, 500, 6
    rng = np.random.default_rng(9)
    lock = (rng.random((Bn, N)) < 0.4).astype(np.uint8)
    masked = ((rng.random((Bn, N)) < 0.3) & (lock == 0)).astype(np.uint8)
    idx, cu = control.compact_active(lock)
    M = len(idx)
    kl, conf = (rng.random(M) * 2e-3).astype(np.float32), rng.random(M).astype(np.float32)
    eps = (rng.random(Bn) * 2e-3).astype(np.float32)
    args = (dev(lock.reshape(-1)), dev(masked.reshape(-1)), dev(idx, torch.int32), dev(cu, torch.int32))
    plain = torch.full((Bn * N,), 7, dtype=torch.uint8, device=DEV)
    if gate > 0:
        B.sl_lock_rule_gated(*args, Bn * N, dev(kl), dev(conf), dev(eps), gate, Bn, N, 0, plain)
    else:
        B.sl_lock_rule(args[0], args[1], args[2], args[3][Bn:], Bn * N, dev(kl), dev(eps), Bn, N, 0, plain)
    out = torch.full((Bn * N,), 7, dtype=torch.uint8, device=DEV)
    tl = torch.zeros(Bn * N, dtype=torch.int32, device=DEV)
    z8, zi = torch.zeros(Bn * N, dtype=torch.uint8, device=DEV), torch.zeros(Bn * N, dtype=torch.int32, device=DEV)
    B.sl_lock_rule_relock(*args, Bn * N, dev(kl), dev(conf), dev(eps), gate, z8, zi, 1.0, t, Bn, N, out, tl)
    torch.cuda.synchronize()
    assert torch.equal(out, plain)
    newly = (out.cpu().numpy() == 1) & (lock.reshape(-1) == 0)
    assert newly.sum() > 0 and np.array_equal(tl.cpu().numpy(), np.where(newly, t, 0))
