"""GPU parity of the whole SureLock step against the oracle, teacher-forced: at every step the
GPU receives the oracle's pre-step state (tokens, masked, lock) and keeps its own K/V cache
and posterior store, so rounding differences cannot compound through decisions.

Checked per step
  exact     active_idx, cu_active
  tolerance logits of the active rows (see gpu_util.logits_tol)
  in situ   KL / conf / argmax against the oracle's fp64 formulas evaluated on the GPU's own
            logits (1e-4 relative on KL), and new_lock / tokens / masked against the oracle's
            control functions applied to the GPU's own kl / conf / argmax (bit-exact)
  decisions sl_lock_test fed the ORACLE's logits must reproduce the oracle's masks and
            unmasked token ids bit-exactly (rows within 1e-6 of the threshold and steps with
            a confidence near-tie at the top-k boundary excluded)
"""
import numpy as np
import pytest
import torch

from oracle import control, model, posterior
from paper_2602_06412_amd import binding as B
from paper_2602_06412_amd import workloads as wl
from tests.gpu_util import DEV, check_logits, dev, oracle_cfg, weights_to_device
from tests.trajectory import near_tie_in_topk, run_oracle, unmask_is_valid

pytestmark = pytest.mark.gpu


def _check_traj(shape, steps, sess, eps, strict_decisions, pre_update=False, gate_m=None):
    Bn, N, V = sess.B, sess.N, shape.vocab
    T = sess.T
    eps_d = dev(np.asarray(eps, dtype=np.float32))
    prev_gpu_logits = None
    for st in steps:
        tokens = dev(st.tokens_in.reshape(-1), torch.int32)
        masked = dev(st.masked_in.reshape(-1).astype(np.uint8))
        lock = dev(st.lock_in.reshape(-1).astype(np.uint8))
        new_lock = torch.full_like(lock, 9)
        lo, hi, k = st.block
        sess.step(tokens, masked, lock, eps_d, st.t, lo, hi, k, new_lock=new_lock)
        torch.cuda.synchronize()
        M = int(sess.cu_active[-1].item())
        assert M == len(st.active_idx), f"t={st.t}"
        assert np.array_equal(sess.cu_active.cpu().numpy(), st.cu_active)
        idx = sess.active_idx[:M].cpu().numpy()
        assert np.array_equal(idx, st.active_idx)
        # logits
        z_gpu = sess.logits_view(st.t)[torch.as_tensor(idx, device=DEV, dtype=torch.long)].to(torch.float64).cpu().numpy()
        check_logits(z_gpu, st.logits, shape.storage, f"t={st.t}")
        # scoring, in situ on the GPU's logits
        kl = sess.kl[:M].cpu().numpy().astype(np.float64)
        conf = sess.conf[:M].cpu().numpy()
        am = sess.argmax[:M].cpu().numpy()
        lp = posterior.log_softmax(z_gpu)
        assert np.array_equal(am, posterior.argmax_lowest(z_gpu))
        assert np.allclose(conf, posterior.max_prob(lp), rtol=2e-6)
        if st.t == 1:
            assert np.all(np.isinf(kl))
        else:
            want = posterior.kl_rows(lp, posterior.log_softmax(prev_gpu_logits[idx]))
            assert np.all(np.abs(kl - want) <= 1e-4 * want + 2e-7), f"t={st.t}"
        prev_full = sess.logits_view(st.t).to(torch.float64).cpu().numpy()
        if prev_gpu_logits is None:
            prev_gpu_logits = prev_full.copy()
        else:
            prev_gpu_logits[idx] = prev_full[idx]
        # device control logic applied to the device's own scores
        want_tok, want_msk, want_lock = st.tokens_in.copy(), st.masked_in.copy().astype(np.uint8), st.lock_in.copy()
        for b in range(Bn):
            r0, r1 = st.cu_active[b], st.cu_active[b + 1]
            pos = st.active_idx[r0:r1] - b * N
            control.update_mask(want_msk[b], want_tok[b], pos, conf[r0:r1], am[r0:r1], lo, hi, k)
            F = control.lock_rule(st.lock_in[b], st.masked_in[b] if pre_update else want_msk[b], pos,
                                  kl[r0:r1].astype(np.float32),
                                  np.maximum(np.float32(0), np.float32(1) - conf[r0:r1]).astype(np.float32),
                                  np.float32(eps[b]), st.t == 1, gate_m=gate_m)
            want_lock[b, F] = 1
        assert np.array_equal(tokens.cpu().numpy().reshape(Bn, N), want_tok), f"t={st.t}"
        assert np.array_equal(masked.cpu().numpy().reshape(Bn, N), want_msk)
        assert np.array_equal(new_lock.cpu().numpy().reshape(Bn, N), want_lock)
        if strict_decisions and not near_tie_in_topk(st, N):
            # fp32 model: the step's own decisions equal the oracle's outright
            assert np.array_equal(want_tok, st.tokens_out), f"t={st.t}"
            safe = np.ones((Bn, N), bool)
            for b in range(Bn):
                r0, r1 = st.cu_active[b], st.cu_active[b + 1]
                near = np.abs(st.kl[r0:r1] - eps[b]) <= 1e-6
                safe[b, (st.active_idx[r0:r1] - b * N)[near]] = False
            assert np.array_equal(want_lock[safe], st.lock_rule_out[safe]), f"t={st.t}"


def _decisions_on_oracle_logits(shape, steps, eps):
    """sl_lock_test on the oracle's logits: masks, indices and unmasked ids bit-exact."""
    T = wl.torch_dtype(shape.storage)
    Bn, N = steps[0].tokens_in.shape
    V = shape.vocab
    prev = torch.zeros(Bn * N, V, dtype=T, device=DEV)
    eps_d = dev(np.asarray(eps, dtype=np.float32))
    n_checked = 0
    for st in steps:
        M = len(st.active_idx)
        cur = dev(st.logits, T)                                  # oracle logits are already on T's grid
        tokens = dev(st.tokens_in.reshape(-1), torch.int32)
        masked = dev(st.masked_in.reshape(-1).astype(np.uint8))
        lock = dev(st.lock_in.reshape(-1).astype(np.uint8))
        idx = torch.zeros(Bn * N, dtype=torch.int32, device=DEV)
        cu = torch.zeros(Bn + 1, dtype=torch.int32, device=DEV)
        B.sl_compact_active(lock, Bn, N, idx, cu)
        kl = torch.zeros(Bn * N, device=DEV); conf = torch.zeros(Bn * N, device=DEV)
        am = torch.zeros(Bn * N, dtype=torch.int32, device=DEV)
        new_lock = torch.zeros_like(lock)
        lo, hi, k = st.block
        B.sl_lock_test(cur, 1, prev, B.dtype_code(T), V, tokens, masked, lock, idx, cu, Bn * N, eps_d, Bn, N,
                       st.t == 1, lo, hi, k, kl, conf, am, new_lock)
        torch.cuda.synchronize()
        assert np.array_equal(idx[:M].cpu().numpy(), st.active_idx)
        assert np.array_equal(am[:M].cpu().numpy(), st.argmax)
        if st.t > 1:
            g = kl[:M].cpu().numpy().astype(np.float64)
            assert np.all(np.abs(g - st.kl) <= 1e-4 * st.kl + 2e-7), f"t={st.t}"
        tok_g, msk_g = tokens.cpu().numpy().reshape(Bn, N), masked.cpu().numpy().reshape(Bn, N)
        assert unmask_is_valid(st, N, tok_g, msk_g), f"t={st.t}"
        if not near_tie_in_topk(st, N):
            assert np.array_equal(tok_g, st.tokens_out), f"t={st.t}"
            assert np.array_equal(msk_g, st.masked_out)
        if np.array_equal(msk_g, st.masked_out):
            safe = np.ones((Bn, N), bool)
            for b in range(Bn):
                r0, r1 = st.cu_active[b], st.cu_active[b + 1]
                near = np.abs(st.kl[r0:r1] - eps[b]) <= 1e-6
                safe[b, (st.active_idx[r0:r1] - b * N)[near]] = False
            assert np.array_equal(new_lock.cpu().numpy().reshape(Bn, N)[safe], st.lock_rule_out[safe]), f"t={st.t}"
            n_checked += 1
        prev[torch.as_tensor(st.active_idx, device=DEV, dtype=torch.long)] = cur
    assert n_checked >= max(1, len(steps) // 4)


def test_c1_tiny_fp32_full_run():
    """Config 1: tiny MDLM fp32, N=128 (32 prompt + 96 mask), T=32, top-3, lock at KL<=1e-3."""
    shape = wl.C1
    w = wl.make_weights(shape, seed=1)
    cfg, w64 = oracle_cfg(shape), wl.weights_to_numpy64(w)
    prompts = [wl.prompt_uniform(7, 32, shape.vocab, shape.mask_id)]
    eps = [1e-3]
    steps = run_oracle(cfg, w64, prompts, 96, 32, 96, eps)
    assert steps[-1].lock_out.sum() > 0 and steps[-1].masked_out.sum() == 0
    sess = B.Session(shape, weights_to_device(w), 1, 128)
    try:
        _check_traj(shape, steps, sess, eps, strict_decisions=True)
    finally:
        sess.close()
    _decisions_on_oracle_logits(shape, steps, eps)


def test_c1_candidates_from_pre_update_mask():
    """The other reading of the candidate line (Alg. 1 prints UpdateMASK first; Sec. 2.1 can be read
    as 'unmasked before this step'): config switch in the library, flag in the oracle; the whole
    config-1 trajectory must agree, and it must differ from the literal reading's."""
    shape = wl.C1
    w = wl.make_weights(shape, seed=1)
    cfg, w64 = oracle_cfg(shape), wl.weights_to_numpy64(w)
    prompts = [wl.prompt_uniform(7, 32, shape.vocab, shape.mask_id)]
    eps = [1e-3]
    steps = run_oracle(cfg, w64, prompts, 96, 32, 96, eps, candidates_pre_update=True)
    literal = run_oracle(cfg, w64, prompts, 96, 32, 96, eps)
    assert any(not np.array_equal(a.lock_out, b.lock_out) for a, b in zip(steps, literal))
    sess = B.Session(shape, weights_to_device(w), 1, 128, candidates_pre_update=True)
    try:
        _check_traj(shape, steps, sess, eps, strict_decisions=True, pre_update=True)
    finally:
        sess.close()


def test_c1_with_confidence_gate():
    """Config 1 with the paper's default gate (only candidates within the 20th percentile of
    uncertainty may lock): the step's own decisions from its own scores equal the oracle's rule
    applied to the same scores at every step, and the gate does change the trajectory."""
    shape = wl.C1
    w = wl.make_weights(shape, seed=1)
    cfg, w64 = oracle_cfg(shape), wl.weights_to_numpy64(w)
    prompts = [wl.prompt_uniform(7, 32, shape.vocab, shape.mask_id)]
    eps = [1e-3]
    ungated = run_oracle(cfg, w64, prompts, 96, 32, 96, eps)
    steps = run_oracle(cfg, w64, prompts, 96, 32, 96, eps, gate_m=20.0)
    assert steps[-1].lock_out.sum() > 0
    assert any(not np.array_equal(a.lock_out, b.lock_out) for a, b in zip(steps, ungated))
    sess = B.Session(shape, weights_to_device(w), 1, 128, gate_percentile=20.0)
    try:
        _check_traj(shape, steps, sess, eps, strict_decisions=False, gate_m=20.0)
    finally:
        sess.close()


def test_c1_lock_disabled_is_full_recompute():
    shape = wl.C1
    w = wl.make_weights(shape, seed=2)
    cfg, w64 = oracle_cfg(shape), wl.weights_to_numpy64(w)
    eps = [-1.0]
    steps = run_oracle(cfg, w64, [wl.prompt_uniform(8, 32, shape.vocab, shape.mask_id)], 96, 8, 96, eps)
    assert all(len(s.active_idx) == 128 for s in steps)
    sess = B.Session(shape, weights_to_device(w), 1, 128)
    try:
        _check_traj(shape, steps, sess, eps, strict_decisions=True)
    finally:
        sess.close()


@pytest.mark.parametrize("shape,Bn,n_p,n_gen,T,block,M_end", [
    (wl.S_BF16, 1, 72, 128, 16, 64, [24]),          # N=200: ragged vs the 64-slot cache padding
    (wl.S_BF16, 3, 40, 96, 12, 96, [16, 50, 136]),   # batch with different M per sequence
    (wl.S_BF16_WIDE, 2, 64, 64, 8, 32, [20, 70]),
    (wl.S_BF16_H64, 2, 30, 70, 10, 70, [10, 33]),     # bf16 on the shape-generic kernels
    (wl.S_BF16, 2, 1000, 100, 5, 100, [40, 300]),     # N = 1100: 18 key tiles, the last one ragged: beyond the thin attention kernel's 16, so the keys are split over workgroups (+ merge)
    (wl.S_BF16_FFN, 1, 40, 56, 8, 56, [12]),          # thin steps whose gate|up + SwiGLU launch is the 256-column weight stream
])
def test_bf16_small_forced_schedule(shape, Bn, n_p, n_gen, T, block, M_end):
    w = wl.make_weights(shape, seed=3, norm_gain_jitter=0.05)
    cfg, w64 = oracle_cfg(shape), wl.weights_to_numpy64(w)
    prompts = [wl.prompt_zipf(20 + b, n_p, shape.vocab, shape.mask_id) for b in range(Bn)]
    eps = [[1e-4, 1e-3, 1e-2][b % 3] for b in range(Bn)]
    steps = run_oracle(cfg, w64, prompts, n_gen, T, block, eps, forced_M_end=M_end, seed=4)
    assert [int(s.cu_active[-1]) for s in steps][-1] < Bn * (n_p + n_gen)
    sess = B.Session(shape, weights_to_device(w), Bn, n_p + n_gen)
    try:
        _check_traj(shape, steps, sess, eps, strict_decisions=False)
    finally:
        sess.close()
    _decisions_on_oracle_logits(shape, steps, eps)


def test_kv_cache_matches_oracle_and_is_permanent():
    shape = wl.S_BF16
    w = wl.make_weights(shape, seed=5)
    cfg, w64 = oracle_cfg(shape), wl.weights_to_numpy64(w)
    n_p, n_gen, T = 40, 64, 8
    N = n_p + n_gen
    steps, states = run_oracle(cfg, w64, [wl.prompt_uniform(1, n_p, shape.vocab, shape.mask_id)], n_gen, T, n_gen,
                               [1e-3], forced_M_end=[30], seed=6, keep_states=True)
    sess = B.Session(shape, weights_to_device(w), 1, N)
    try:
        eps_d = dev(np.array([1e-3], dtype=np.float32))
        snaps = []
        for st in steps:
            lo, hi, k = st.block
            sess.step(dev(st.tokens_in.reshape(-1), torch.int32), dev(st.masked_in.reshape(-1).astype(np.uint8)),
                      dev(st.lock_in.reshape(-1).astype(np.uint8)), eps_d, st.t, lo, hi, k)
            snaps.append([tuple(t.clone() for t in sess.kv_read(l)) for l in range(shape.n_layers)])
        torch.cuda.synchronize()
        # final cache equals the oracle's (bf16 grid: allow one spacing on a few elements)
        for l in range(shape.n_layers):
            kg, vg = (t[0].to(torch.float64).cpu().numpy() for t in snaps[-1][l])
            for got, want in ((kg, states[0].Kc[l]), (vg, states[0].Vc[l])):
                err = np.abs(got - want)
                assert np.all(err <= np.maximum(2e-2, 2.0 ** (np.floor(np.log2(np.maximum(np.abs(want), 1e-30))) - 7)))
                if l == 0:          # first layer: inputs are exact, only accumulation order differs
                    assert np.mean(err > 0) < 0.05
        # rows locked before step t are byte-identical in the cache before and after step t
        for ti in range(1, T):
            locked = np.flatnonzero(steps[ti].lock_in[0])
            assert len(locked) > 0
            li = torch.as_tensor(locked, device=DEV, dtype=torch.long)
            for l in range(shape.n_layers):
                for a, b_ in zip(snaps[ti][l], snaps[ti - 1][l]):
                    assert torch.equal(a[0, li], b_[0, li])
    finally:
        sess.close()


@pytest.mark.parametrize("scale,what", [(3.0e5, "beyond the half range"), (2.0e-6, "below the normal half range")])
def test_v_cache_container_at_the_ends_of_its_range(scale, what):
    """The bf16 route keeps V, rounded to bf16, in a half-precision container (attention multiplies it by
    half-precision probabilities).  With the V projection scaled by 3e5 many |V| exceed 65504: they are stored
    saturated, never as infinity (a zero probability times infinity would be NaN), and the logits stay
    finite.  Scaled by 2e-6 all |V| fall below the smallest normal half 2^-14: they are kept to the container's
    absolute resolution 2^-24, not flushed to zero.  Every value between those ends is held exactly, which
    the other cache tests check."""
    shape = wl.S_BF16
    w = wl.make_weights(shape, seed=5)
    for lw in w["layers"]:
        lw["wv"] = (lw["wv"].float() * scale).to(lw["wv"].dtype)
    cfg, w64 = oracle_cfg(shape), wl.weights_to_numpy64(w)
    N = 96
    tokens_np = wl.prompt_uniform(2, N, shape.vocab, shape.mask_id)
    sess = B.Session(shape, weights_to_device(w), 1, N)
    try:
        zero = torch.zeros(N, dtype=torch.uint8, device=DEV)
        sess.step(dev(tokens_np, torch.int32), zero.clone(), zero, dev(np.array([1e-3], dtype=np.float32)), 1, 0, N, 0)
        torch.cuda.synchronize()
        vg = sess.kv_read(0)[1][0].to(torch.float64).cpu().numpy()
        # layer 0's V from the definition: rnd(rnd(rmsnorm(emb)) Wv^T)
        L0 = w64["layers"][0]
        h = cfg.rnd(model.rmsnorm(w64["emb"][tokens_np], L0["attn_norm"], cfg.rms_eps))
        v = cfg.rnd(h @ L0["wv"].T).reshape(N, cfg.n_heads, cfg.d_head)
        assert np.isfinite(vg).all()
        assert torch.isfinite(sess.logits_view(1).float()).all()
        if scale > 1:
            big = np.abs(v) > 65504
            assert big.mean() > 0.05, "the case must reach the end of the range"
            # 65504 read back as bf16 is 65536 (the nearest bf16 value)
            assert np.all(np.abs(vg[big]) == 65536.0) and np.all(np.sign(vg[big]) == np.sign(v[big]))
            ok = ~big & (np.abs(v) < 6.0e4)
            err = np.abs(vg[ok] - v[ok])
            assert np.all(err <= 2.0 ** (np.floor(np.log2(np.maximum(np.abs(v[ok]), 1e-30))) - 7))
        else:
            assert (np.abs(v) < 2.0 ** -14).all() and (np.abs(v) > 2.0 ** -22).mean() > 0.5
            # container resolution 2^-24 (half a step each way), plus the bf16 rounding of the read-back and the
            # one-spacing slack of an fp32 sum that sits on a bf16 rounding boundary
            err = np.abs(vg - v)
            assert np.all(err <= 2.0 ** -25 + 2.0 ** (np.floor(np.log2(np.maximum(np.abs(v), 1e-30))) - 7))
            assert (vg != 0).mean() > 0.9
    finally:
        sess.close()


@pytest.mark.parametrize("N", [7680, 7650])
def test_longest_sequence(N):
    """The step at its longest sequence (7680 slots, the limit of UpdateMASK's selection; 120 key tiles; and 7650
    slots, whose last key tile holds 34 slots and 30 masked ones): two
    sequences of a one-layer bf16 model.  Step 1 computes every row (480 (row tile, head) workgroups: the
    three-per-CU attention kernel walks all 120 tiles); step 2 computes 200 + 40 rows (the pipelined kernel with
    the keys split over 64 workgroups per pair and the merge launch).  The oracle's attention costs M x N, so it
    runs the block for sampled rows only, against the cache the GPU holds for the other slots (whose rows are
    checked the same way when sampled): their K/V rows and their logits."""
    shape = wl.Shape("small-bf16-1layer", 1, 512, 4, 128, 1536, 4160, "bf16")
    Bn = 2
    w = wl.make_weights(shape, seed=9, norm_gain_jitter=0.05)
    cfg, w64 = oracle_cfg(shape), wl.weights_to_numpy64(w)
    R = Bn * N
    tokens_np = wl.prompt_zipf(31, R, shape.vocab, shape.mask_id)
    sess = B.Session(shape, weights_to_device(w), Bn, N)
    rng = np.random.default_rng(2)
    try:
        tokens = dev(tokens_np, torch.int32)
        eps = dev(np.full(Bn, 1e-3, dtype=np.float32))
        zero = torch.zeros(R, dtype=torch.uint8, device=DEV)
        per_seq = [np.arange(N), np.arange(N)]
        for t, counts in ((1, (N, N)), (2, (200, 40))):
            per_seq = [a if m == len(a) else a[wl.active_positions(70 + m, len(a), m)] for a, m in zip(per_seq, counts)]
            active = np.concatenate([b * N + a for b, a in enumerate(per_seq)])
            M = len(active)
            lock = dev(wl.lock_mask_from_active(R, active))
            sess.step(tokens, zero.clone(), lock, eps, t, 0, N, 0, m_upper=M, new_lock=torch.zeros_like(lock))
            torch.cuda.synchronize()
            assert int(sess.cu_active[-1].item()) == M
            assert np.array_equal(sess.active_idx[:M].cpu().numpy(), active)
            kg, vg = (x.to(torch.float64).cpu().numpy() for x in sess.kv_read(0))
            for b in range(Bn):
                a = per_seq[b]
                pos = np.unique(np.concatenate([rng.choice(a, size=6, replace=False), [a[0], a[-1]]]))
                Kc, Vc = kg[b].copy(), vg[b].copy()
                x = model.layer_active(cfg, w64["layers"][0], w64["emb"][tokens_np[b * N + pos]], pos, Kc, Vc)
                for got, want in ((kg[b][pos], Kc[pos]), (vg[b][pos], Vc[pos])):
                    err = np.abs(got - want)
                    assert np.all(err <= 2.0 ** (np.floor(np.log2(np.maximum(np.abs(want), 1e-30))) - 7) + 1e-6)
                z = model.lm_head(cfg, w64, x)
                rows = torch.as_tensor(b * N + pos, device=DEV, dtype=torch.long)
                check_logits(sess.logits_view(t)[rows].double().cpu().numpy(), z, shape.storage, f"N={N} t={t} sequence {b}")
    finally:
        sess.close()


def test_m_upper_tight_and_errors():
    shape = wl.C1
    w = weights_to_device(wl.make_weights(shape, seed=1))
    sess = B.Session(shape, w, 1, 128)
    try:
        lock = np.zeros(128, dtype=np.uint8); lock[::2] = 1
        tokens = dev(wl.prompt_uniform(3, 128, shape.vocab, shape.mask_id), torch.int32)
        masked = dev(np.zeros(128, dtype=np.uint8))
        eps_d = dev(np.array([1e-3], dtype=np.float32))
        sess.step(tokens, masked, dev(lock), eps_d, 1, 0, 128, 0, m_upper=128)
        za = sess.logits_view(1).clone()
        sess.step(tokens, masked, dev(lock), eps_d, 1, 0, 128, 0, m_upper=64)     # exactly M
        torch.cuda.synchronize()
        assert torch.equal(za[1::2], sess.logits_view(1)[1::2])
        for bad in (dict(t=0), dict(m_upper=0), dict(m_upper=129), dict(block_hi=129)):
            kw = dict(t=1, block_lo=0, block_hi=128, k=0, m_upper=128); kw.update(bad)
            with pytest.raises(B.SureLockError) as e:
                B.sl_surelock_step(sess.ctx, tokens, masked, dev(lock), eps_d, kw["t"], kw["block_lo"], kw["block_hi"],
                                   kw["k"], kw["m_upper"], sess.active_idx, sess.cu_active, sess.kl, sess.conf,
                                   sess.argmax, dev(lock), sess.workspace)
            assert e.value.status == B.SL_EINVAL
        small = torch.empty(256, dtype=torch.uint8, device=DEV)
        with pytest.raises(B.SureLockError) as e:
            B.sl_surelock_step(sess.ctx, tokens, masked, dev(lock), eps_d, 1, 0, 128, 0, 128, sess.active_idx,
                               sess.cu_active, sess.kl, sess.conf, sess.argmax, dev(lock), small)
        assert e.value.status == B.SL_ENOSPC
    finally:
        sess.close()


def test_out_of_range_token_ids_are_clamped():
    """Token ids are device data the library cannot validate on the host; ids outside the
    vocabulary read the nearest table row instead of memory outside the table."""
    shape = wl.C1
    w = weights_to_device(wl.make_weights(shape, seed=1))
    sess = B.Session(shape, w, 1, 128)
    try:
        lock = dev(np.zeros(128, dtype=np.uint8))
        masked = dev(np.zeros(128, dtype=np.uint8))
        eps_d = dev(np.array([1e-3], dtype=np.float32))
        tok = wl.prompt_uniform(3, 128, shape.vocab, shape.mask_id).astype(np.int64)
        bad, ok = tok.copy(), tok.copy()
        bad[5], ok[5] = shape.vocab + 12345, shape.vocab - 1
        bad[9], ok[9] = -3, 0
        bad[17], ok[17] = 2 ** 31 - 1, shape.vocab - 1
        sess.step(dev(ok, torch.int32), masked, lock, eps_d, 1, 0, 128, 0, m_upper=128)
        z_ok = sess.logits_view(1).clone()
        sess.step(dev(bad, torch.int32), masked, lock, eps_d, 1, 0, 128, 0, m_upper=128)
        torch.cuda.synchronize()
        assert torch.equal(z_ok, sess.logits_view(1))
    finally:
        sess.close()


def test_m_upper_too_small_is_contained():
    """A bound below the true number of active rows: the first m_upper active rows are processed exactly
    as in a step with a valid bound, nothing is written past m_upper entries of the packed arrays, no
    position beyond them is unmasked or locked, and cu_active reports the true counts."""
    shape = wl.C1
    w = weights_to_device(wl.make_weights(shape, seed=1))
    Bn, N, mu = 2, 64, 40
    sess = B.Session(shape, w, Bn, N)
    try:
        lock = np.zeros((Bn, N), dtype=np.uint8); lock[0, ::4] = 1; lock[1, 1::3] = 1
        true_M = int((lock == 0).sum())
        assert true_M > mu
        tok0 = np.stack([wl.prompt_uniform(3 + b, N, shape.vocab, shape.mask_id) for b in range(Bn)])
        masked0 = (1 - lock).astype(np.uint8)                 # every active slot can be unmasked
        eps_d = dev(np.array([1e30, 1e30], dtype=np.float32))   # every unmasked active row would lock at t = 2
        out = {}
        for name, bound in (("ok", Bn * N), ("small", mu)):
            tokens, masked = dev(tok0.reshape(-1), torch.int32), dev(masked0.reshape(-1))
            for t in (1, 2):
                for buf in (sess.active_idx, sess.argmax):
                    buf.fill_(-7)
                sess.kl.fill_(-7.0); sess.conf.fill_(-7.0)
                new_lock = torch.full((Bn * N,), 9, dtype=torch.uint8, device=DEV)
                sess.step(tokens, masked, dev(lock.reshape(-1)), eps_d, t, 0, N, 5 if t == 2 else 0, m_upper=bound,
                          new_lock=new_lock)
            torch.cuda.synchronize()
            out[name] = [x.cpu().numpy().copy() for x in (sess.active_idx, sess.cu_active, sess.kl, sess.conf, sess.argmax,
                                                          tokens, masked, new_lock)]
        idx_ok, cu_ok, kl_ok, conf_ok, am_ok, tok_ok, msk_ok, lock_ok = out["ok"]
        idx, cu, kl, conf, am, tok, msk, nl = out["small"]
        assert np.array_equal(cu, cu_ok) and cu[-1] == true_M
        assert np.array_equal(idx[:mu], idx_ok[:mu]) and np.all(idx[mu:] == -7)
        assert np.all(am[mu:] == -7) and np.all(kl[mu:] == -7.0) and np.all(conf[mu:] == -7.0)
        assert np.array_equal(am[:mu], am_ok[:mu])
        beyond = idx_ok[mu:true_M]                            # flat ids of the active rows the bound cut off
        assert np.array_equal(tok[beyond], tok0.reshape(-1)[beyond]) and np.all(msk[beyond] == 1)
        assert np.all(nl[beyond] != 1)                        # never locked (left as the caller's buffer held them)
        changed = np.flatnonzero(msk != masked0.reshape(-1))
        assert len(changed) > 0 and set(changed) <= set(idx_ok[:mu].tolist())
    finally:
        sess.close()


@pytest.mark.parametrize("shape", [wl.C1, wl.S_BF16])
def test_sequences_without_active_rows(shape):
    """Degenerate batches: a sequence whose positions are all locked contributes no row (its neighbour's
    logits are bit for bit those of the same sequence stepped alone, with the same row bound), and a step
    in which nothing is active at all computes nothing, unmasks nothing and returns the lock mask unchanged."""
    w = weights_to_device(wl.make_weights(shape, seed=2))
    N, mu = 96, 48
    eps2, eps1 = dev(np.array([1e-3, 1e-3], dtype=np.float32)), dev(np.array([1e-3], dtype=np.float32))
    tok = np.stack([wl.prompt_uniform(5 + b, N, shape.vocab, shape.mask_id) for b in range(2)])
    lock = np.ones((2, N), dtype=np.uint8)
    act = np.sort(np.random.default_rng(1).choice(N, size=37, replace=False))
    lock[1, act] = 0                                              # sequence 0: nothing active; sequence 1: 37 rows
    masked = np.zeros((2, N), dtype=np.uint8); masked[1, act[-5:]] = 1
    s2, s1 = B.Session(shape, w, 2, N), B.Session(shape, w, 1, N)
    try:
        # step 1: all of sequence 1 (its K/V and first posteriors), nothing of sequence 0, under the same row bound
        # in both sessions, so that both run the same launches
        z8 = torch.zeros(2 * N, dtype=torch.uint8, device=DEV)
        lock_first = torch.cat([torch.ones(N, dtype=torch.uint8, device=DEV), z8[:N]])
        s2.step(dev(tok.reshape(-1), torch.int32), z8.clone(), lock_first, eps2, 1, 0, N, 0, m_upper=N)
        s1.step(dev(tok[1], torch.int32), z8[:N].clone(), z8[:N].clone(), eps1, 1, 0, N, 0, m_upper=N)
        torch.cuda.synchronize()
        assert s2.cu_active.cpu().tolist() == [0, 0, N]
        assert torch.equal(s2.logits_view(1)[N:], s1.logits_view(1))
        t2, m2 = dev(tok.reshape(-1), torch.int32), dev(masked.reshape(-1))
        t1, m1 = dev(tok[1], torch.int32), dev(masked[1])
        nl2 = torch.full((2 * N,), 9, dtype=torch.uint8, device=DEV)
        nl1 = torch.full((N,), 9, dtype=torch.uint8, device=DEV)
        s2.step(t2, m2, dev(lock.reshape(-1)), eps2, 2, 0, N, 2, m_upper=mu, new_lock=nl2)
        s1.step(t1, m1, dev(lock[1]), eps1, 2, 0, N, 2, m_upper=mu, new_lock=nl1)
        torch.cuda.synchronize()
        assert s2.cu_active.cpu().tolist() == [0, 0, 37] and s1.cu_active.cpu().tolist() == [0, 37]
        assert np.array_equal(s2.active_idx[:37].cpu().numpy(), N + act)
        rows2 = torch.as_tensor(N + act, device=DEV, dtype=torch.long)
        rows1 = torch.as_tensor(act, device=DEV, dtype=torch.long)
        assert torch.equal(s2.logits_view(2)[rows2], s1.logits_view(2)[rows1])
        assert torch.equal(s2.kl[:37], s1.kl[:37]) and torch.equal(s2.argmax[:37], s1.argmax[:37])
        assert torch.equal(nl2[N:], nl1) and torch.all(nl2[:N] == 1)
        assert torch.equal(t2[N:], t1) and torch.equal(m2[N:], m1) and torch.equal(t2[:N].cpu(), torch.as_tensor(tok[0], dtype=torch.int32))
        assert int(m1.sum().item()) == 3                          # two of the five masked slots were unmasked
        # nothing active at all
        all_locked = torch.ones(2 * N, dtype=torch.uint8, device=DEV)
        kv_before, post_before = s2.kv.clone(), s2.post.clone()
        t3, m3 = t2.clone(), m2.clone()
        nl3 = torch.full((2 * N,), 9, dtype=torch.uint8, device=DEV)
        s2.step(t3, m3, all_locked, eps2, 3, 0, N, 2, m_upper=mu, new_lock=nl3)
        torch.cuda.synchronize()
        assert s2.cu_active.cpu().tolist() == [0, 0, 0]
        assert torch.all(nl3 == 1) and torch.equal(t3, t2) and torch.equal(m3, m2)
        assert torch.equal(s2.kv, kv_before) and torch.equal(s2.post, post_before)
    finally:
        s2.close()
        s1.close()


def test_largest_batch():
    """SL_MAX_BATCH = 255 sequences of 64 slots in one step (16320 packed rows, then a ragged step in which
    every sequence keeps a different number of active rows, some none): sampled sequences against the oracle's
    full forward of that sequence alone, the packed row ranges against the definition."""
    from oracle import model
    shape, Bn, N = wl.S_BF16, 255, 64
    w = wl.make_weights(shape, seed=7, norm_gain_jitter=0.05)
    cfg, w64 = oracle_cfg(shape), wl.weights_to_numpy64(w)
    tok = np.stack([wl.prompt_uniform(100 + b, N, shape.vocab, shape.mask_id) for b in range(Bn)])
    sess = B.Session(shape, weights_to_device(w), Bn, N)
    try:
        eps = dev(np.full(Bn, 1e-3, dtype=np.float32))
        z8 = torch.zeros(Bn * N, dtype=torch.uint8, device=DEV)
        tokens = dev(tok.reshape(-1), torch.int32)
        sess.step(tokens, z8.clone(), z8.clone(), eps, 1, 0, N, 0, m_upper=Bn * N, new_lock=torch.zeros_like(z8))
        torch.cuda.synchronize()
        assert sess.cu_active.cpu().tolist() == [b * N for b in range(Bn + 1)]
        for b in (0, 127, 254):
            z, _, _ = model.forward_full(cfg, w64, tok[b])
            z_gpu = sess.logits_view(1)[b * N:(b + 1) * N].double().cpu().numpy()
            check_logits(z_gpu, z, "bf16", f"B=255 step 1, sequence {b}")
        # ragged: sequence b keeps b % 9 of its rows active (every ninth sequence none)
        lock = np.ones((Bn, N), dtype=np.uint8)
        rng = np.random.default_rng(3)
        for b in range(Bn):
            lock[b, rng.choice(N, size=b % 9, replace=False)] = 0
        active, cu = control.compact_active(lock)
        M = len(active)
        sess.step(tokens, z8.clone(), dev(lock.reshape(-1)), eps, 2, 0, N, 0, m_upper=M, new_lock=torch.zeros_like(z8))
        torch.cuda.synchronize()
        assert np.array_equal(sess.cu_active.cpu().numpy(), cu)
        assert np.array_equal(sess.active_idx[:M].cpu().numpy(), active)
        # unchanged tokens and a cache that already holds this forward's K/V: the restricted rows reproduce step 1
        rows = torch.as_tensor(active, device=DEV, dtype=torch.long)
        d = (sess.logits_view(2)[rows].float() - sess.logits_view(1)[rows].float()).abs()
        assert float(d.max()) <= 0.0625 and float((d > 0).float().mean()) < 0.25
        assert torch.all(sess.kl[:M] < 1e-3)
    finally:
        sess.close()
