"""Algorithmic-FLOP model (Sec. 2.4; test infrastructure).

Only GEMMs are counted: Q/K/V/Out projections, QK^T and AV, and the FFN.
"""


def f_base_step(L, B, N_b, d, H, d_h, H_kv, d_ff):
    """Baseline FLOPs of one step for one batch (the 'Baseline' equation)."""
    return L * (4 * B * H * N_b * N_b * d_h        # QK^T + AV
                + 2 * B * N_b * d * d              # Q
                + 2 * B * N_b * d * d              # Out
                + 4 * B * N_b * d * H_kv * d_h     # K, V
                + 6 * B * N_b * d * d_ff)          # FFN


def f_prop_step(M_tb, L, B, N_b, d, H, d_h, H_kv, d_ff):
    """SureLock FLOPs of one step: |A_t,b| / (B N_b) of the baseline
    (the 'SureLock' equation)."""
    return M_tb / (B * N_b) * f_base_step(L, B, N_b, d, H, d_h, H_kv, d_ff)


def f_base_per_position(S, L, N_b, d, H, d_h, H_kv, d_ff):
    """Per-token-position baseline FLOPs summed over S steps.  This is the
    normalisation under which the F_base column of the continuation table
    (LLaDA-8B-Base, WikiText-103) is reproduced: F^t_base,b / T_b, times S."""
    return S * f_base_step(L, 1, N_b, d, H, d_h, H_kv, d_ff) / N_b


def r_bar(M, N_b, B):
    """Micro-averaged active ratio: sum_b sum_t M_{t,b} / sum_b sum_t B N_b
    (Experiment 1).  M: list over batches of lists over steps; N_b: list."""
    num = sum(sum(m) for m in M)
    den = sum(len(m) * B * n for m, n in zip(M, N_b))
    return num / den
