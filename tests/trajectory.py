"""Oracle trajectories for the teacher-forced GPU parity tests (not collected by pytest).

run_oracle() drives oracle.sampler for B independent sequences and records, per step, the
state BEFORE the step (tokens, masked, lock) and everything the step produced, batched the
way the C ABI sees it (flat row ids b*N + i, sequences concatenated)."""
from dataclasses import dataclass

import numpy as np

from oracle import sampler
from paper_2602_06412_amd import workloads as wl


@dataclass
class BatchStep:
    t: int
    tokens_in: np.ndarray      # [B, N]
    masked_in: np.ndarray      # [B, N]
    lock_in: np.ndarray        # [B, N]
    block: tuple               # (lo, hi, k)
    active_idx: np.ndarray     # [M] flat ids
    cu_active: np.ndarray      # [B+1]
    logits: np.ndarray         # [M, V]
    kl: np.ndarray
    conf: np.ndarray
    argmax: np.ndarray
    tokens_out: np.ndarray
    masked_out: np.ndarray
    lock_rule_out: np.ndarray  # lock_in | F_t  (what the KL rule alone gives)
    lock_out: np.ndarray       # lock mask carried to the next step (rule and/or forced)
    d_last_in: np.ndarray = None   # [B, N] fp32, only for runs with selection


def run_oracle(cfg, w64, prompts, n_gen, T, block_len, eps, forced_M_end=None, seed=0, keep_states=False,
               candidates_pre_update=False, gate_m=None, select_k=None):
    """prompts: list of B int arrays (same length); eps: list of B thresholds.
    forced_M_end: None -> the KL rule drives the mask; else a list of per-sequence final
    active counts: a seeded priority force-locks eligible rows so M falls linearly, and the
    rule's F_t is recorded only."""
    Bn = len(prompts)
    n_p = len(prompts[0])
    N = n_p + n_gen
    sched = sampler.block_schedule(n_p, n_gen, block_len, T)
    states = [sampler.init_state(cfg, w64, p, n_gen) for p in prompts]
    hooks = [None] * Bn
    if forced_M_end is not None:
        for b in range(Bn):
            pri = np.random.default_rng(seed * 1000 + b).permutation(N)
            target = wl.linear_m_schedule(N, forced_M_end[b], T)

            def hook(st, rec, pri=pri, target=target):
                nxt = target[st.t] if st.t < len(target) else target[-1]
                return wl.forced_lock_positions(pri, st.lock, st.masked, int((st.lock == 0).sum()) - nxt)
            hooks[b] = hook
    steps = []
    for t in range(T):
        lo, hi, k = sched[t]
        pre = [(s.tokens.copy(), s.masked.copy(), s.lock.copy()) for s in states]
        d_last_in = np.stack([s.d_last.copy() for s in states])
        recs = [sampler.surelock_step(cfg, w64, states[b], eps[b], lo, hi, k, forced_lock=hooks[b],
                                      kl_drives_lock=forced_M_end is None,
                                      candidates_pre_update=candidates_pre_update, gate_m=gate_m,
                                      select_k=select_k) for b in range(Bn)]
        idx = np.concatenate([r.active_pos + b * N for b, r in enumerate(recs)])
        cu = np.concatenate([[0], np.cumsum([len(r.active_pos) for r in recs])])
        rule = np.stack([p[2].copy() for p in pre])
        for b, r in enumerate(recs):
            rule[b, r.F] = 1
        steps.append(BatchStep(
            t=t + 1, tokens_in=np.stack([p[0] for p in pre]), masked_in=np.stack([p[1] for p in pre]),
            lock_in=np.stack([p[2] for p in pre]), block=(lo, hi, k), active_idx=idx, cu_active=cu,
            logits=np.concatenate([r.logits for r in recs]), kl=np.concatenate([r.kl for r in recs]),
            conf=np.concatenate([r.conf for r in recs]), argmax=np.concatenate([r.argmax for r in recs]),
            tokens_out=np.stack([s.tokens.copy() for s in states]),
            masked_out=np.stack([s.masked.copy() for s in states]),
            lock_rule_out=rule, lock_out=np.stack([s.lock.copy() for s in states]), d_last_in=d_last_in))
    return (steps, states) if keep_states else steps


def near_tie_in_topk(step, N, rel=1e-5):
    """True if, in some sequence, the k-th and (k+1)-th most confident eligible rows are
    closer than `rel` relative: then either choice is valid and the step is skipped by the
    exact-token comparison."""
    lo, hi, k = step.block
    Bn = step.tokens_in.shape[0]
    for b in range(Bn):
        r0, r1 = step.cu_active[b], step.cu_active[b + 1]
        pos = step.active_idx[r0:r1] - b * N
        c = sorted((float(step.conf[r0 + j]) for j in range(r1 - r0)
                    if step.masked_in[b, pos[j]] and lo <= pos[j] < hi), reverse=True)
        if k < len(c) and k > 0 and abs(c[k - 1] - c[k]) <= rel * c[k - 1]:
            return True
    return False


def unmask_is_valid(step, N, tokens_gpu, masked_gpu, rel=1e-5):
    """The GPU's UpdateMASK result is a valid confidence-ordered top-k of the oracle's own
    confidences: exactly min(k, #eligible) eligible positions unmasked per sequence, none of
    them less confident (beyond `rel`) than an eligible position left masked, each given its
    row's argmax token, and nothing else changed.  Without near-ties this is equality."""
    lo, hi, k = step.block
    Bn = step.tokens_in.shape[0]
    for b in range(Bn):
        r0, r1 = step.cu_active[b], step.cu_active[b + 1]
        pos = step.active_idx[r0:r1] - b * N
        elig = {int(pos[j]): r0 + j for j in range(r1 - r0) if step.masked_in[b, pos[j]] and lo <= pos[j] < hi}
        changed = set(np.flatnonzero(masked_gpu[b] != step.masked_in[b]).tolist())
        if not changed <= set(elig) or len(changed) != min(k, len(elig)):
            return False
        if np.any(masked_gpu[b][list(changed)] != 0):
            return False
        for i in range(N):
            want = step.argmax[elig[i]] if i in changed else step.tokens_in[b, i]
            if tokens_gpu[b, i] != want:
                return False
        left = [step.conf[r] for i, r in elig.items() if i not in changed]
        took = [step.conf[r] for i, r in elig.items() if i in changed]
        if left and took and min(took) < max(left) * (1 - rel):
            return False
    return True


@dataclass
class UnlockStep:
    """One step of a run with optional unlocking, batched like BatchStep; *_in is the state before
    the step, lock_mid the lock mask after the step's lock update (what the probe sees), *_out the
    state after the probe and the unlock rule (equal to *_mid on steps without a probe)."""
    base: BatchStep
    t_lock_in: np.ndarray      # [B, N]
    relocked_in: np.ndarray
    cool_in: np.ndarray
    lock_mid: np.ndarray
    t_lock_mid: np.ndarray
    probe: list                # per sequence ProbeRecord or None
    lock_out: np.ndarray
    relocked_out: np.ndarray
    cool_out: np.ndarray


def run_oracle_unlock(cfg, w64, prompts, n_gen, T, block_len, eps, prm, forced_M_end=None, seed=0):
    """As run_oracle, with oracle.sampler.UnlockParams prm switched on."""
    Bn = len(prompts)
    n_p = len(prompts[0])
    N = n_p + n_gen
    sched = sampler.block_schedule(n_p, n_gen, block_len, T)
    states = [sampler.init_state(cfg, w64, p, n_gen) for p in prompts]
    hooks = [None] * Bn
    mids = [None] * Bn
    if forced_M_end is not None:
        for b in range(Bn):
            pri = np.random.default_rng(seed * 1000 + b).permutation(N)
            target = wl.linear_m_schedule(N, forced_M_end[b], T)

            def hook(st, rec, pri=pri, target=target):
                nxt = target[st.t] if st.t < len(target) else target[-1]
                return wl.forced_lock_positions(pri, st.lock, st.masked, int((st.lock == 0).sum()) - nxt)
            hooks[b] = hook
    out = []
    for t in range(T):
        lo, hi, k = sched[t]
        pre = [(s.tokens.copy(), s.masked.copy(), s.lock.copy(), s.lock_step.copy(), s.relocked.copy(),
                s.cool_until.copy()) for s in states]
        recs = [sampler.surelock_step(cfg, w64, states[b], eps[b], lo, hi, k, forced_lock=hooks[b],
                                      kl_drives_lock=forced_M_end is None, unlock=prm) for b in range(Bn)]
        idx = np.concatenate([r.active_pos + b * N for b, r in enumerate(recs)])
        cu = np.concatenate([[0], np.cumsum([len(r.active_pos) for r in recs])])
        rule = np.stack([p[2].copy() for p in pre])
        mid = np.stack([p[2].copy() for p in pre])
        for b, r in enumerate(recs):
            rule[b, r.F] = 1
            mid[b, (r.F if forced_M_end is None else [])] = 1
            mid[b, r.forced] = 1
        base = BatchStep(
            t=t + 1, tokens_in=np.stack([p[0] for p in pre]), masked_in=np.stack([p[1] for p in pre]),
            lock_in=np.stack([p[2] for p in pre]), block=(lo, hi, k), active_idx=idx, cu_active=cu,
            logits=np.concatenate([r.logits for r in recs]), kl=np.concatenate([r.kl for r in recs]),
            conf=np.concatenate([r.conf for r in recs]), argmax=np.concatenate([r.argmax for r in recs]),
            tokens_out=np.stack([s.tokens.copy() for s in states]),
            masked_out=np.stack([s.masked.copy() for s in states]),
            lock_rule_out=rule, lock_out=np.stack([s.lock.copy() for s in states]))
        out.append(UnlockStep(
            base=base, t_lock_in=np.stack([p[3] for p in pre]), relocked_in=np.stack([p[4] for p in pre]),
            cool_in=np.stack([p[5] for p in pre]), lock_mid=mid,
            t_lock_mid=np.stack([s.lock_step.copy() for s in states]), probe=[r.probe for r in recs],
            lock_out=np.stack([s.lock.copy() for s in states]),
            relocked_out=np.stack([s.relocked.copy() for s in states]),
            cool_out=np.stack([s.cool_until.copy() for s in states])))
    return out
