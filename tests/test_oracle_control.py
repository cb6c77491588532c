"""Pins of the oracle's index-set / mask logic and FLOP model: brute force over
all small patterns, library percentiles, and the values the paper prints."""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import control, flops


def test_compaction_all_patterns_up_to_6():
    for N in range(1, 7):
        for bits in itertools.product([0, 1], repeat=N):
            lock = np.array([bits, bits[::-1]], dtype=np.uint8)     # B = 2
            idx, cu = control.compact_active(lock)
            want = sorted(b * N + i for b in range(2) for i in range(N) if lock[b, i] == 0)
            assert list(idx) == want
            assert list(cu) == [0, N - sum(bits), 2 * (N - sum(bits))]


def test_update_mask_topk_ties_and_block():
    #           pos: 0    1    2    3    4    5
    masked = np.array([0, 1, 1, 1, 1, 1], dtype=np.uint8)
    tokens = np.array([7, 99, 99, 99, 99, 99])
    pos = np.array([0, 1, 2, 3, 4, 5])
    conf = np.array([0.99, 0.5, 0.9, 0.9, 0.95, 0.2], dtype=np.float32)
    amax = np.array([10, 11, 12, 13, 14, 15])
    # block [1, 4): position 4 (highest conf) is outside; 2 and 3 tie -> lower position first
    got = control.update_mask(masked, tokens, pos, conf, amax, 1, 4, 1)
    assert got == [2] and tokens[2] == 12 and masked[2] == 0 and masked[3] == 1
    got = control.update_mask(masked, tokens, pos, conf, amax, 1, 4, 5)   # k larger than what is left
    assert got == [3, 1] and list(masked) == [0, 0, 0, 0, 1, 1]
    assert list(tokens) == [7, 11, 12, 13, 99, 99]
    assert control.update_mask(masked, tokens, pos, conf, amax, 1, 4, 3) == []


def test_update_mask_against_sorted_brute_force():
    rng = np.random.default_rng(0)
    for trial in range(50):
        N = 12
        masked = rng.integers(0, 2, N).astype(np.uint8)
        conf = rng.integers(0, 4, N).astype(np.float32) / 4       # many ties
        amax = rng.integers(0, 100, N)
        lo, hi, k = 2, 10, int(rng.integers(0, 5))
        order = sorted([i for i in range(lo, hi) if masked[i]], key=lambda i: (-conf[i], i))[:k]
        m2, t2 = masked.copy(), np.full(N, -1)
        got = control.update_mask(m2, t2, np.arange(N), conf, amax, lo, hi, k)
        assert got == order
        for i in range(N):
            assert m2[i] == (0 if i in order else masked[i])
            assert t2[i] == (amax[i] if i in order else -1)


@pytest.mark.parametrize("m", [10, 20, 40, 50, 100])
def test_percentile_nearest_rank_matches_library(m):
    rng = np.random.default_rng(m)
    for n in (1, 2, 5, 10, 37):
        v = rng.random(n)
        assert control.percentile_nearest_rank(v, m) == np.percentile(v, m, method="inverted_cdf")


def test_lock_rule_all_patterns():
    N = 5
    rng = np.random.default_rng(1)
    for lockbits in itertools.product([0, 1], repeat=N):
        for maskbits in itertools.product([0, 1], repeat=N):
            lock = np.array(lockbits, dtype=np.uint8)
            masked = np.array(maskbits, dtype=np.uint8)
            if np.any(lock & masked):
                continue                        # a masked slot is never locked
            pos = np.flatnonzero(lock == 0)
            D = rng.random(len(pos)).astype(np.float32)
            u = rng.random(len(pos)).astype(np.float32)
            Z = {int(p) for p in pos if not masked[p]}
            F = control.lock_rule(lock, masked, pos, D, u, np.float32(0.5), first_step=False)
            assert set(F) <= Z and F == sorted(F)
            assert set(F) == {int(p) for r, p in enumerate(pos) if p in Z and D[r] <= 0.5}
            assert control.lock_rule(lock, masked, pos, D, u, np.float32(0.5), first_step=True) == []
            assert set(control.lock_rule(lock, masked, pos, D, u, math.inf, False)) == Z
            assert control.lock_rule(lock, masked, pos, D, u, np.float32(-1.0), False) == []
            # boundary: D == eps locks (the rule is <=)
            if len(pos):
                assert (int(pos[0]) in control.lock_rule(lock, masked, pos, D, u, D[0], False)) == (int(pos[0]) in Z)
            # gate: only candidates whose u is at most the m-th percentile over Z
            G = control.lock_rule(lock, masked, pos, D, u, math.inf, False, gate_m=20)
            if Z:
                uz = sorted(float(u[r]) for r, p in enumerate(pos) if p in Z)
                th = uz[max(1, math.ceil(0.2 * len(uz))) - 1]
                assert set(G) == {int(p) for r, p in enumerate(pos) if p in Z and u[r] <= th}
                assert len(G) >= 1


def test_flops_table_values_printed_in_the_paper():
    path = os.path.join(os.path.dirname(__file__), "golden", "flops_continuation_table.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 8
    for n_gen, steps, printed in rows:
        n_gen, steps, printed = int(n_gen), int(steps), float(printed)
        got = flops.f_base_per_position(steps, 32, 64 + n_gen, 4096, 32, 128, 32, 12288)
        assert abs(got / printed - 1) < 6e-4, (n_gen, steps, got, printed)   # 4 printed digits


def test_flops_structure():
    kw = dict(L=32, B=4, N_b=320, d=4096, H=32, d_h=128, H_kv=32, d_ff=12288)
    base = flops.f_base_step(**kw)
    # per-row GEMM terms at LLaDA-8B shape: 2d^2 + 2d^2 + 4d^2 + 6 d d_ff = 436,207,616
    per_row_layer = base / (32 * 4 * 320) - 4 * 32 * 320 * 128
    assert per_row_layer == 436207616
    assert flops.f_prop_step(4 * 320, **kw) == base
    assert flops.f_prop_step(320, **kw) == base / 4
    assert flops.r_bar([[4, 2], [8, 8]], [2, 4], 2) == (6 + 16) / (2 * 2 * 2 + 2 * 2 * 4)
