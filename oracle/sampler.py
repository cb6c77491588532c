"""Algorithm 1 (SureLock) and the plain sampler, one sequence at a time
(test infrastructure; a batch is an independent loop over sequences).

State follows the 'State' lines of Alg. 1: lock, the per-layer K/V caches,
the previous posteriors, the masked set and the frozen block input x_hat.
Decisions that a floating-point value takes (ranking by confidence, D <= eps,
the percentile gate) are taken on the value rounded to fp32.  The paper fixes no
precision for them (Sec. 2.2 states D_t <= eps over real numbers), and a
decision has to be taken in ONE precision on both sides of a comparison to be
comparable at all: fp32 is what a scoring pass over fp32-accumulated
log-probabilities yields.  The values themselves (log-softmax, KL, confidence)
stay fp64 up to that point, so the cast can flip a decision only where the
fp64 value lies within one fp32 spacing of the threshold (relative 6e-8; the
KL accuracy bound of the GPU tests, 1e-4 relative, is three orders of magnitude
wider and those tests exclude |D - eps| <= 1e-6 from mask equality anyway).
"""
from dataclasses import dataclass, field

import numpy as np

from . import control, model, posterior, sampling


@dataclass
class State:
    tokens: np.ndarray            # [N] int64, mask_id on still-masked slots
    masked: np.ndarray            # [N] uint8, 1 = prediction target (M_t)
    lock: np.ndarray              # [N] uint8, monotone
    Kc: list                      # L x [N, H, d_h]
    Vc: list
    prev_lp: np.ndarray           # [N, V] log p_{t-1}; rows of locked slots keep log p_{t*}
    x_hat: np.ndarray             # [N, d] frozen block input (bookkeeping only)
    lock_step: np.ndarray         # [N] int64, step at which the slot locked (0 = never)
    t: int = 0
    relocked: np.ndarray = None   # [N] uint8, 1 = was unlocked at least once (stricter re-lock)
    cool_until: np.ndarray = None # [N] int64, the slot cannot lock while t <= cool_until
    d_last: np.ndarray = None     # [N] float32, the KL the slot scored when last computed (+inf before)


@dataclass(frozen=True)
class UnlockParams:
    """Parameters of App. 'Optional Unlocking'."""
    period: int                   # P: the probe runs after every P-th step
    m: float                      # theta_t = m-th percentile of u over the active rows
    eps_unlock: float
    d_interval: int               # a slot stays locked for more than this many steps
    d_cool: int                   # steps after an unlock during which the slot cannot re-lock
    rho: float = 1.0              # re-lock threshold rho * eps, rho <= 1


@dataclass
class ProbeRecord:
    pos: np.ndarray               # probed (locked) positions, ascending
    logits: np.ndarray            # [R, V] proxy logits
    u: np.ndarray                 # proxy uncertainty 1 - max p^
    conf: np.ndarray
    D: np.ndarray                 # KL(p^_t || p_{t*})
    unlocked: list                # positions the rule unlocks


@dataclass
class StepRecord:
    t: int
    active_pos: np.ndarray        # A_t, ascending
    logits: np.ndarray            # [M, V] in active order
    kl: np.ndarray                # [M] D_t (inf at t = 1)
    u: np.ndarray                 # [M] 1 - max p
    conf: np.ndarray              # [M] max p
    argmax: np.ndarray            # [M]
    unmasked: list                # positions unmasked at this step, selection order
    F: list                       # positions the KL rule locks at this step
    forced: list = field(default_factory=list)   # positions locked by a forced schedule
    probe: ProbeRecord = None     # set on the steps where the unlock probe ran
    write_id: np.ndarray = None   # [M] the token UpdateMASK would write per row (argmax, or the draw at tau > 0)


def init_state(cfg, weights, prompt_tokens, n_gen):
    """Alg. 1 state initialisation: nothing locked, caches empty, no previous
    posterior, the n_gen generation slots masked, x_hat = prompt embeddings."""
    n_p = len(prompt_tokens)
    N = n_p + n_gen
    tokens = np.concatenate([np.asarray(prompt_tokens, dtype=np.int64),
                             np.full(n_gen, cfg.mask_id, dtype=np.int64)])
    masked = np.zeros(N, dtype=np.uint8)
    masked[n_p:] = 1
    shape = (N, cfg.n_heads, cfg.d_head)
    x_hat = np.zeros((N, cfg.d_model))
    x_hat[:n_p] = weights["emb"][tokens[:n_p]]
    return State(tokens=tokens, masked=masked, lock=np.zeros(N, dtype=np.uint8),
                 Kc=[np.full(shape, np.nan) for _ in range(cfg.n_layers)],
                 Vc=[np.full(shape, np.nan) for _ in range(cfg.n_layers)],
                 prev_lp=np.full((N, cfg.vocab), np.nan), x_hat=x_hat,
                 lock_step=np.zeros(N, dtype=np.int64), relocked=np.zeros(N, dtype=np.uint8),
                 cool_until=np.zeros(N, dtype=np.int64), d_last=np.full(N, np.inf, dtype=np.float32))


def surelock_step(cfg, weights, st, eps, block_lo, block_hi, k,
                  gate_m=None, candidates_pre_update=False, forced_lock=None,
                  kl_drives_lock=True, unlock=None, select_k=None, temperature=0.0, seed=0, seq_index=0):
    """One iteration of the loop of Alg. 1, in the paper's order.

    eps < 0 can never be met by a KL (>= 0), which turns locking off.
    forced_lock(st, record) -> list of positions, if given, is a workload hook
    (not part of the method) that locks further positions after the rule ran;
    with kl_drives_lock=False the rule's F_t is recorded but not applied.
    unlock: UnlockParams or None.  When given, re-locking obeys the cool-down and
    the stricter threshold, and after every unlock.period-th step the read-only
    probe and the unlock rule of App. 'Optional Unlocking' run (unlock_probe).
    select_k: None or the fraction k of Exp-5's combined setting: from step 2 on
    only control.select_rows' choice among the non-locked positions is computed;
    a skipped position keeps its K/V, its posterior and its lock state, and its
    next KL is taken against the posterior of the step it was last computed at.
    temperature > 0 (App. on sampling temperature): UpdateMASK still ranks by the
    raw-posterior confidence but writes a token drawn from softmax(z / temperature)
    (sampling.sample_token, keyed by seed, the step and the flat row id
    seq_index * N + position); scores and the lock test are untouched.
    """
    st.t += 1
    t = st.t
    # active / locked sets
    A = np.flatnonzero(st.lock == 0)
    if select_k is not None and t > 1:
        A = np.asarray(control.select_rows(A, st.masked, st.d_last, block_lo, block_hi, select_k), dtype=np.int64)
    tokens_in = st.tokens.copy()
    # restricted forward on the active rows; live K/V overwrite their cache rows
    z = model.forward_active(cfg, weights, st.tokens, A, st.Kc, st.Vc)
    lp = posterior.log_softmax(z)
    conf = posterior.max_prob(lp)
    amax = posterior.argmax_lowest(z)
    # unmasking
    masked_before = st.masked.copy()
    write_id = amax.copy()
    if temperature > 0:
        N = len(st.tokens)
        for r, p in enumerate(A):
            if st.masked[p] and block_lo <= p < block_hi:
                write_id[r] = sampling.sample_token(z[r], temperature, seed, t, seq_index * N + int(p))
    unmasked = control.update_mask(st.masked, st.tokens, A,
                                   conf.astype(np.float32), write_id, block_lo, block_hi, k)
    # score
    u = posterior.uncertainty(lp)
    if t > 1:
        D = posterior.kl_rows(lp, st.prev_lp[A])
    else:
        D = np.full(len(A), np.inf)
    # candidates and lock rule
    m_for_Z = masked_before if candidates_pre_update else st.masked
    F = control.lock_rule(st.lock, m_for_Z, A, D.astype(np.float32), u.astype(np.float32),
                          np.float32(eps), first_step=(t == 1), gate_m=gate_m,
                          relocked=st.relocked if unlock is not None else None,
                          cool_until=st.cool_until if unlock is not None else None,
                          rho=unlock.rho if unlock is not None else 1.0, t=t)
    rec = StepRecord(t=t, active_pos=A, logits=z, kl=D, u=u, conf=conf, argmax=amax,
                     unmasked=unmasked, F=F, write_id=write_id)
    # posteriors of the active rows become p_{t-1}; locked rows keep p_{t*}
    st.prev_lp[A] = lp
    st.d_last[A] = np.maximum(D, 0.0).astype(np.float32)       # KL >= 0; rounding may leave -1e-17
    to_lock = list(F) if kl_drives_lock else []
    if forced_lock is not None:
        rec.forced = [int(p) for p in forced_lock(st, rec)]
        to_lock = sorted(set(to_lock) | set(rec.forced))
    for p in to_lock:
        # K/V of p were written into Kc/Vc by this step's forward and are never
        # written again: that is the cache commit of the lock line.
        st.lock[p] = 1
        st.lock_step[p] = t
        st.x_hat[p] = weights["emb"][tokens_in[p]]
    if unlock is not None and t % unlock.period == 0:
        rec.probe = unlock_probe(cfg, weights, st, unlock, u.astype(np.float32))
    return rec


def unlock_probe(cfg, weights, st, prm, u_active):
    """App. 'Optional Unlocking', run after step st.t is complete.

    The proxy is the network itself restricted to the locked rows: their
    current tokens go through all blocks with queries only (keys and values of
    every slot, their own included, are read from the cache and nothing is
    written, so the step just taken is unchanged), then the LM head.  This
    gives u~ = 1 - max p^ and D~ = KL(p^_t || p_{t*}) against the posterior
    kept from the step the slot locked at.  The unlock rule then clears the
    lock of the chosen slots, marks them for the stricter re-lock threshold and
    starts their cool-down; they are active again from step t + 1, where their
    K/V rows are overwritten (that is the invalidation) and their KL is taken
    against the last posterior kept for them, p_{t*}.
    u_active: fp32 uncertainties of this step's active rows (theta_t is their
    percentile).  Values that decide are rounded to fp32 first.
    """
    t = st.t
    Lpos = np.flatnonzero(st.lock == 1)
    if len(Lpos) == 0:
        return ProbeRecord(pos=Lpos, logits=np.zeros((0, cfg.vocab)), u=np.zeros(0), conf=np.zeros(0),
                           D=np.zeros(0), unlocked=[])
    z = model.forward_active(cfg, weights, st.tokens, Lpos, st.Kc, st.Vc, write_cache=False)
    lp = posterior.log_softmax(z)
    u = posterior.uncertainty(lp)
    D = posterior.kl_rows(lp, st.prev_lp[Lpos])
    unlocked = control.unlock_rule(st.lock_step, Lpos, u.astype(np.float32), D.astype(np.float32), u_active,
                                   prm.m, np.float32(prm.eps_unlock), t, prm.d_interval)
    for p in unlocked:
        st.lock[p] = 0
        st.relocked[p] = 1
        st.cool_until[p] = t + prm.d_cool
    return ProbeRecord(pos=Lpos, logits=z, u=u, conf=posterior.max_prob(lp), D=D, unlocked=unlocked)


def baseline_step(cfg, weights, tokens, masked, block_lo, block_hi, k):
    """One step of the same sampler without locking: full recompute of all N
    positions, then UpdateMASK.  Returns (logits [N, V], K list, V list, unmasked)."""
    z, Ks, Vs = model.forward_full(cfg, weights, tokens)
    lp = posterior.log_softmax(z)
    conf = posterior.max_prob(lp).astype(np.float32)
    amax = posterior.argmax_lowest(z)
    unmasked = control.update_mask(masked, tokens, np.arange(len(tokens)), conf, amax,
                                   block_lo, block_hi, k)
    return z, Ks, Vs, unmasked


def block_schedule(n_prompt, n_gen, block_len, T):
    """Semi-autoregressive schedule: the generation region is cut into blocks of
    block_len slots, each block gets T / n_blocks consecutive steps and
    block_len / steps_per_block tokens are unmasked per step.
    Returns a list over steps of (block_lo, block_hi, k)."""
    n_blocks = n_gen // block_len
    assert n_blocks * block_len == n_gen and T % n_blocks == 0
    spb = T // n_blocks
    assert block_len % spb == 0
    k = block_len // spb
    out = []
    for t in range(T):
        b = t // spb
        out.append((n_prompt + b * block_len, n_prompt + (b + 1) * block_len, k))
    return out
