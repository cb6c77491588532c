"""Index-set and mask logic of the oracle (test infrastructure).

Alg. 1: active set (the line defining A_t and L_t), UpdateMASK, locking
candidates Z_t, the optional confidence gate and the lock rule F_t.
Plain Python / NumPy loops; integer results are exact.
"""
import math

import numpy as np


def compact_active(lock):
    """A_t = {i : lock_i = 0} for a batch.  lock: [B, N] (0/1).

    Returns (active_idx, cu_active): active_idx lists the flat row ids b*N+i of
    the unlocked positions, sequences in order and positions ascending inside
    each sequence; cu_active[b] is the number of active rows before sequence b
    (exclusive prefix sum), cu_active[B] the total M.
    """
    lock = np.asarray(lock)
    B, N = lock.shape
    idx, cu = [], [0]
    for b in range(B):
        for i in range(N):
            if not lock[b, i]:
                idx.append(b * N + i)
        cu.append(len(idx))
    return np.asarray(idx, dtype=np.int64), np.asarray(cu, dtype=np.int64)


def update_mask(masked, tokens, pos, conf, argmax_id, block_lo, block_hi, k):
    """UpdateMASK for one sequence (confidence-ordered unmasking, temperature 0).

    Among the still-masked positions inside the current semi-autoregressive
    block [block_lo, block_hi), take the k with the highest posterior maximum
    ``conf`` (ties: lowest position first), write the argmax token there and
    clear the masked flag.  pos / conf / argmax_id are parallel arrays over the
    active rows of this sequence (every masked position is active, because only
    unmasked positions can ever lock).  masked and tokens are updated in place.
    Returns the list of positions unmasked, in selection order.
    """
    cand = [(-float(conf[r]), int(pos[r]), r) for r in range(len(pos))
            if masked[pos[r]] and block_lo <= pos[r] < block_hi]
    cand.sort()
    chosen = []
    for _, p, r in cand[:k]:
        tokens[p] = int(argmax_id[r])
        masked[p] = 0
        chosen.append(p)
    return chosen


def percentile_nearest_rank(values, m):
    """The m-th percentile by nearest rank: the ceil(m/100 * n)-th smallest value
    (at least the 1st).  The paper leaves the interpolation open; this is the
    reading taken."""
    v = sorted(float(x) for x in values)
    if not v:
        return -math.inf
    rank = max(1, math.ceil(m * len(v) / 100.0))
    return v[rank - 1]


def lock_rule(lock, masked_for_candidates, pos, D, u, eps, first_step, gate_m=None,
              relocked=None, cool_until=None, rho=1.0, t=None):
    """Z_t = active and unmasked; F_t = {i in Z_t : u_i <= theta_m and D_i <= eps}.

    pos / D / u are parallel arrays over the active rows of one sequence.
    ``masked_for_candidates`` is the masked flag array the candidate set is
    built from (Alg. 1 places UpdateMASK before the candidate line, so the
    literal reading passes the post-update flags).  At the first step D is
    +inf, so nothing locks.  gate_m=None disables the optional confidence gate.
    With relocked / cool_until given (App. 'Optional Unlocking'): a position that
    was unlocked before needs D_i <= rho * eps (the product formed in fp32, like
    the comparison) and cannot lock while t <= cool_until_i.
    Returns the sorted list of positions to lock (F_t); lock is not modified.
    """
    Z = [r for r in range(len(pos)) if not lock[pos[r]] and not masked_for_candidates[pos[r]]]
    if first_step:
        return []
    theta = math.inf
    if gate_m is not None:
        theta = percentile_nearest_rank([u[r] for r in Z], gate_m)
    def thresh(p):
        if relocked is not None and relocked[p]:
            return np.float32(rho) * np.float32(eps)
        return eps

    def cooled(p):
        return cool_until is None or t > cool_until[p]

    F = [int(pos[r]) for r in Z if u[r] <= theta and D[r] <= thresh(pos[r]) and cooled(pos[r])]
    return sorted(F)


def unlock_rule(lock_step, pos_probe, u_probe, D_probe, u_active, m, eps_unlock, t, d_interval):
    """The unlock condition of App. 'Optional Unlocking' (its displayed equation)
    for one sequence: with theta_t the m-th percentile (nearest rank, as for the
    gate) of the uncertainty u_t over the ACTIVE rows of step t, a probed locked
    position i is unlocked iff
        u~_i > theta_t  and  D~_i > eps_unlock  and  t - t*_i > D_interval,
    all three strictly (the sentence before the equation says 'any', the
    equation joins them with 'and'; the equation is followed).  With no active
    row theta_t = -inf.  pos_probe / u_probe / D_probe are parallel arrays over
    the probed rows, lock_step[i] = t*_i.  Returns the sorted positions to unlock.
    """
    theta = percentile_nearest_rank(u_active, m)
    out = [int(p) for r, p in enumerate(pos_probe)
           if u_probe[r] > theta and D_probe[r] > eps_unlock and t - int(lock_step[p]) > d_interval]
    return sorted(out)


def select_rows(pos_active, masked, d_last, block_lo, block_hi, k_frac):
    """Selection-based sparsification on top of the lock mask (Exp-5, the combined
    setting: a fixed fraction k of the positions not yet locked is computed per step).

    The paper's surrogate does not say which positions; the reading taken: of the n
    active positions of a sequence, ceil(k * n) are computed.  The still-masked
    positions of the current block always are (they must stay decodable; they may
    exceed the budget); the rest of the budget goes to the other active positions in
    decreasing order of the KL they scored when last computed (d_last, fp32, +inf
    before any score), ties to the lower position.  Returns the sorted positions to
    compute.
    """
    pos_active = [int(p) for p in pos_active]
    n = len(pos_active)
    budget = min(n, math.ceil(float(k_frac) * n))
    must = [p for p in pos_active if masked[p] and block_lo <= p < block_hi]
    must_set = set(must)
    rest = sorted((p for p in pos_active if p not in must_set), key=lambda p: (-float(d_last[p]), p))
    take = must + rest[:max(0, budget - len(must))]
    return sorted(take)
